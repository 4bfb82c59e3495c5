// f16-storage instantiations of the packed-filter window kernel (stride-1 layers, channel-innermost input).
#include "pwin_kernel.h"

namespace convfwd {

//                                     DT       R  S  KW WN TMB NBW AD LBT
#define PW(...) PwinCfg<CONV_F16, __VA_ARGS__>

void register_pwin_f16(std::vector<Variant>& out)
{
    // 3x3
    pwin_register<PW(3, 3, 4, 1, 2, 3, 9, 6)>(out);  // M64 N96  C64, 4 waves: 64x96 wave tiles, 192 slab positions
    pwin_register<PW(3, 3, 4, 1, 2, 2, 9, 5)>(out);  // M64 N64  C64, 4 waves
    pwin_register<PW(3, 3, 4, 2, 2, 3, 9, 5)>(out);  // M64 N192 C64, 8 waves
    pwin_register<PW(3, 3, 2, 2, 2, 3, 9, 8)>(out);  // M64 N192 C32, 4 waves
    pwin_register<PW(3, 3, 8, 1, 2, 3, 9, 6)>(out);  // M64 N96  C128, 8 waves (two per SIMD)
    pwin_register<PW(3, 3, 8, 1, 2, 3, 3, 6)>(out);  // the same with a filter ring of 3 taps
    pwin_register<PW(3, 3, 8, 1, 2, 2, 3, 5)>(out);  // M64 N64  C128, 8 waves
    // 5x5
    pwin_register<PW(5, 5, 2, 2, 2, 4, 5, 9)>(out);  // M64 N256 C32, 4 waves: 64x128 wave tiles, 576 slab positions
    pwin_register<PW(5, 5, 2, 2, 2, 3, 5, 8)>(out);  // M64 N192 C32, 4 waves
    pwin_register<PW(5, 5, 2, 2, 2, 4, 5, 10, true)>(out);  // M64 N256 C32 with the conflict-free row pitch
    pwin_register<PW(5, 5, 2, 2, 2, 2, 5, 6)>(out);         // M64 N128 C32, 4 waves: small enough for two workgroups per CU
}

}  // namespace convfwd
