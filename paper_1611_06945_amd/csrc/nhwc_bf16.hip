// bf16-storage instantiations of the channel-innermost implicit-GEMM kernel.
#include "nhwc_kernel.h"

namespace convfwd {

#define NH16CFG(WM, WN, BM, BN, TK) IgemmCfg<CONV_BF16, 32, WM, WN, BM, BN, TK, true, MODE_GATHER>

void register_nhwc_bf16(std::vector<Variant>& out)
{
    const std::initializer_list<int> sk_all = {1, 2, 4, 8}, sk_few = {1, 2, 4};
    nhwc_register<NH16CFG(2, 2, 2, 2, 64)>(out, sk_few);   // M128 N128
    nhwc_register<NH16CFG(2, 2, 2, 2, 32)>(out, sk_few);   // M128 N128
    nhwc_register<NH16CFG(2, 2, 2, 1, 64)>(out, sk_all);   // M128 N64
    nhwc_register<NH16CFG(2, 2, 1, 2, 64)>(out, sk_all);   // M64  N128
    nhwc_register<NH16CFG(2, 2, 1, 2, 32)>(out, sk_all);   // M64  N128
    nhwc_register<NH16CFG(2, 2, 1, 1, 64)>(out, sk_all);   // M64  N64
    nhwc_register<NH16CFG(2, 2, 1, 1, 32)>(out, sk_all);   // M64  N64
    nhwc_register<NH16CFG(1, 4, 1, 1, 64)>(out, sk_all);   // M32  N128
    nhwc_register<NH16CFG(1, 4, 3, 1, 64)>(out, sk_few);   // M96  N128
    // eight waves per workgroup: the same tiles with more waves to cover the latency of the staging loads
    nhwc_register<NH16CFG(2, 4, 2, 1, 64)>(out, sk_few);   // M128 N128, waves of 64x32
    nhwc_register<NH16CFG(4, 2, 1, 2, 64)>(out, sk_few);   // M128 N128, waves of 32x64
    nhwc_register<NH16CFG(2, 4, 1, 1, 64)>(out, sk_few);   // M64  N128, waves of 32x32
}

}  // namespace convfwd
