// bf16-storage instantiations of the packed-filter window kernel (stride-1 layers, channel-innermost input).
#include "pwin_kernel.h"

namespace convfwd {

//                                     DT       R  S  KW WN TMB NBW AD LBT
#define PW(...) PwinCfg<CONV_BF16, __VA_ARGS__>

void register_pwin_bf16(std::vector<Variant>& out)
{
    // 3x3
    pwin_register<PW(3, 3, 4, 1, 2, 3, 9, 6)>(out);  // M64 N96  C64, 4 waves: 64x96 wave tiles, 192 slab positions
    pwin_register<PW(3, 3, 4, 1, 2, 2, 9, 5)>(out);  // M64 N64  C64, 4 waves
    pwin_register<PW(3, 3, 4, 2, 2, 3, 9, 5)>(out);  // M64 N192 C64, 8 waves
    pwin_register<PW(3, 3, 2, 2, 2, 3, 9, 8)>(out);  // M64 N192 C32, 4 waves
    pwin_register<PW(3, 3, 8, 1, 2, 3, 9, 6)>(out);  // M64 N96  C128, 8 waves (two per SIMD)
    pwin_register<PW(3, 3, 8, 1, 2, 3, 3, 6)>(out);  // the same with a filter ring of 3 taps
    pwin_register<PW(3, 3, 8, 1, 2, 2, 3, 5)>(out);  // M64 N64  C128, 8 waves
    // 32-row tiles for small operations (a few hundred to a few thousand pixels): little to exchange between the
    // channel-waves and many workgroups; chunk sizes for every channel count that is a multiple of 16, slab sizes for
    // short and long rows
    pwin_register<PW(3, 3, 8, 1, 1, 1, 3, 4)>(out);  // M32 N32 C128, 8 waves, 128 slab positions
    pwin_register<PW(3, 3, 8, 1, 1, 2, 3, 5)>(out);  // M32 N64 C128, 8 waves, 160
    pwin_register<PW(3, 3, 4, 1, 1, 1, 9, 4)>(out);  // M32 N32 C64,  4 waves, 128
    pwin_register<PW(3, 3, 4, 1, 1, 1, 9, 8)>(out);  // M32 N32 C64,  4 waves, 256 (rows of 28 and 56 pixels)
    pwin_register<PW(3, 3, 4, 1, 1, 2, 9, 8)>(out);  // M32 N64 C64,  4 waves, 256
    pwin_register<PW(3, 3, 2, 1, 1, 1, 9, 4)>(out);  // M32 N32 C32,  2 waves, 128
    pwin_register<PW(3, 3, 2, 2, 1, 1, 9, 4)>(out);  // M32 N64 C32,  4 waves, 256
    pwin_register<PW(3, 3, 2, 2, 1, 2, 9, 8)>(out);  // M32 N128 C32, 4 waves, 512 (rows of 56 pixels)
    pwin_register<PW(3, 3, 1, 2, 1, 1, 9, 2)>(out);  // M32 N64 C16,  2 waves, 128 (channel counts like 112 and 144)
    pwin_register<PW(3, 3, 1, 4, 1, 1, 9, 2)>(out);  // M32 N128 C16, 4 waves, 256
    // 5x5
    pwin_register<PW(5, 5, 2, 2, 2, 4, 5, 9)>(out);  // M64 N256 C32, 4 waves: 64x128 wave tiles, 576 slab positions
    pwin_register<PW(5, 5, 2, 2, 2, 3, 5, 8)>(out);  // M64 N192 C32, 4 waves
    pwin_register<PW(5, 5, 2, 2, 2, 4, 5, 10, true)>(out);  // M64 N256 C32 with the conflict-free row pitch
    pwin_register<PW(5, 5, 2, 2, 2, 2, 5, 6)>(out);         // M64 N128 C32, 4 waves: small enough for two workgroups per CU
    pwin_register<PW(5, 5, 2, 1, 1, 1, 5, 6)>(out);         // M32 N32 C32,  2 waves, 192 slab positions
    pwin_register<PW(5, 5, 2, 2, 1, 1, 5, 5)>(out);         // M32 N64 C32,  4 waves, 320
    pwin_register<PW(5, 5, 1, 2, 1, 1, 5, 3)>(out);         // M32 N64 C16,  2 waves, 192
    pwin_register<PW(5, 5, 1, 4, 1, 1, 5, 3)>(out);         // M32 N128 C16, 4 waves, 384
}

}  // namespace convfwd
