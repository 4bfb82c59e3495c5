// fp32 instantiations of the window-reuse kernel (stride-1 layers whose padded image slab fits in LDS).
#include "wconv_kernel.h"

namespace convfwd {

//                       DT        R  S  CPL TMB NB  LB
#define WCFG(R, S, CPL, TMB, NB, LB, WN) WconvCfg<CONV_F32, R, S, CPL, TMB, NB, LB, WN>

void register_wconv_f32(std::vector<Variant>& out)
{
    const std::initializer_list<int> sk = {1, 2, 4, 8};
    // 3x3: 13x13 outputs (169 -> 11 pixel blocks), 14x14 (196 -> 13 blocks)
    wconv_register<WCFG(3, 3, 1, 2, 11, 2, 2)>(out, sk);
    wconv_register<WCFG(3, 3, 1, 1, 11, 2, 2)>(out, sk);
    wconv_register<WCFG(3, 3, 1, 2, 11, 4, 1)>(out, sk);
    wconv_register<WCFG(3, 3, 1, 1, 11, 4, 1)>(out, sk);
    wconv_register<WCFG(3, 3, 1, 2, 13, 2, 2)>(out, sk);
    wconv_register<WCFG(3, 3, 1, 1, 13, 2, 2)>(out, sk);
    // pixel tiles of half a 13x13 or 14x14 image: twice the workgroups for small batches without a split reduction
    wconv_register<WCFG(3, 3, 1, 1, 6, 2, 2)>(out, sk);
}

}  // namespace convfwd
