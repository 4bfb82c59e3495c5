// Instantiations of the fp32 window kernel whose waves split the channels of a chunk (stride-1 3x3 and 5x5 layers).
#include "pwin32_kernel.h"

namespace convfwd {

//                        R  S  KW WN TMB NBW CPW SLOTS
#define P32(...) Pwin32Cfg<__VA_ARGS__>

void register_pwin32_f32(std::vector<Variant>& out)
{
    // 3x3 (9 steps per channel pair: 2 steps of look-ahead, 3 register sets)
    pwin32_register<P32(3, 3, 8, 1, 1, 1, 2, 128, 2)>(out);   // M32 N32  C16, 8 waves
    pwin32_register<P32(3, 3, 16, 1, 1, 1, 2, 128, 2)>(out);  // M32 N32  C32, 16 waves
    pwin32_register<P32(3, 3, 4, 1, 1, 1, 4, 128, 2)>(out);   // M32 N32  C16, 4 waves
    pwin32_register<P32(3, 3, 8, 1, 2, 1, 2, 128, 2)>(out);   // M64 N32  C16, 8 waves
    pwin32_register<P32(3, 3, 8, 1, 1, 2, 2, 256, 2)>(out);   // M32 N64  C16, 8 waves
    pwin32_register<P32(3, 3, 8, 1, 1, 1, 2, 256, 2)>(out);   // M32 N32  C16, 8 waves, longer rows
    pwin32_register<P32(3, 3, 4, 2, 2, 3, 4, 512, 1)>(out);   // M64 N192 C16, 8 waves
    // 5x5 (25 steps per channel pair: 4 steps of look-ahead, 5 register sets)
    pwin32_register<P32(5, 5, 4, 1, 1, 1, 2, 256, 4)>(out);   // M32 N32  C8,  4 waves
    pwin32_register<P32(5, 5, 8, 1, 1, 1, 2, 256, 4)>(out);   // M32 N32  C16, 8 waves
    pwin32_register<P32(5, 5, 4, 1, 2, 2, 2, 512, 4)>(out);   // M64 N64  C8,  4 waves
    pwin32_register<P32(5, 5, 4, 2, 2, 2, 2, 512, 4)>(out);   // M64 N128 C8,  8 waves
}

}  // namespace convfwd
