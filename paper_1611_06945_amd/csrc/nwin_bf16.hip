// bf16-storage instantiations of the channel-innermost window-reuse kernel (stride-1 layers, band of output rows per workgroup).
#include "nwin_kernel.h"

namespace convfwd {

//                                          DT        R  S  KW WM TMB WN NBW LBT
#define NW(R, S, KW, WM, TMB, WN, NBW, LBT) NwinCfg<CONV_BF16, R, S, KW, WM, TMB, WN, NBW, LBT>

void register_nwin_bf16(std::vector<Variant>& out)
{
    const std::initializer_list<int> sk = {1, 2, 4};
    // 3x3
    nwin_register<NW(3, 3, 4, 1, 1, 2, 3, 3)>(out, sk);  // M32 N192 C64, 8 waves
    nwin_register<NW(3, 3, 2, 1, 1, 2, 3, 3)>(out, sk);  // M32 N192 C32, 4 waves
    nwin_register<NW(3, 3, 2, 2, 1, 2, 3, 2)>(out, sk);  // M64 N192 C32, 8 waves
    nwin_register<NW(3, 3, 2, 1, 2, 2, 3, 3)>(out, sk);  // M64 N192 C32, 4 waves, 64x96 wave tiles
    // 5x5
    nwin_register<NW(5, 5, 2, 1, 1, 2, 3, 5)>(out, sk);  // M32 N192 C32, 4 waves
    nwin_register<NW(5, 5, 1, 2, 1, 2, 3, 3)>(out, sk);  // M64 N192 C16, 4 waves
    // 5x5, larger pixel tiles: every workgroup refetches its filter slab, so more pixels per slab
    nwin_register<NW(5, 5, 1, 1, 1, 8, 3, 4)>(out, sk);  // M32 N768 C16, 8 waves (27x27 image whole)
    nwin_register<NW(5, 5, 1, 2, 1, 4, 3, 2)>(out, sk);  // M64 N384 C16, 8 waves
}

}  // namespace convfwd
