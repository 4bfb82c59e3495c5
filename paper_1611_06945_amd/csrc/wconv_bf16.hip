// bf16-storage instantiations of the 16-bit window-reuse kernel (stride-1 layers, band of output rows per workgroup).
#include "wconv16_kernel.h"

namespace convfwd {

//                                        DT      R  S  KW WM TMB WN NBW LBT
#define W16(R, S, KW, WM, TMB, WN, NBW, LBT) Wconv16Cfg<CONV_BF16, R, S, KW, WM, TMB, WN, NBW, LBT>
#define W16I(R, S, KW, WM, TMB, WN, NBW, LBT, LBN) Wconv16Cfg<CONV_BF16, R, S, KW, WM, TMB, WN, NBW, LBT, LBN>

void register_wconv_bf16(std::vector<Variant>& out)
{
    const std::initializer_list<int> sk = {1, 2, 4};
    // 3x3
    wconv16_register<W16(3, 3, 2, 1, 1, 2, 3, 4)>(out, sk);  // M32 N192 C32, 4 waves
    wconv16_register<W16(3, 3, 4, 1, 1, 2, 3, 3)>(out, sk);  // M32 N192 C64, 8 waves
    wconv16_register<W16(3, 3, 2, 2, 1, 2, 3, 2)>(out, sk);  // M64 N192 C32, 8 waves
    wconv16_register<W16(3, 3, 2, 1, 2, 2, 3, 3)>(out, sk);  // M64 N192 C32, 4 waves, 64x96 wave tiles
    // 3x3, whole image per workgroup staged through a raw LDS copy (16-byte global loads)
    wconv16_register<W16I(3, 3, 4, 1, 1, 2, 3, 3, 4)>(out, sk);  // M32 N192 C64, 8 waves
    wconv16_register<W16I(3, 3, 2, 1, 1, 2, 3, 4, 4)>(out, sk);  // M32 N192 C32, 4 waves
    wconv16_register<W16I(3, 3, 2, 2, 1, 2, 3, 2, 2)>(out, sk);  // M64 N192 C32, 8 waves
    // 5x5
    wconv16_register<W16(5, 5, 2, 1, 1, 2, 3, 5)>(out, sk);  // M32 N192 C32, 4 waves
    wconv16_register<W16(5, 5, 1, 2, 1, 2, 3, 3)>(out, sk);  // M64 N192 C16, 4 waves
}

}  // namespace convfwd
