// bf16-storage instantiations of the scalar-offset implicit-GEMM kernel (bf16 MFMA, fp32 accumulate).
#include "ugemm_kernel.h"

namespace convfwd {

#define U16CFG(MB, WM, WN, BM, BN, TK, AVEC) IgemmCfg<CONV_BF16, MB, WM, WN, BM, BN, TK, AVEC, MODE_GATHER>

void register_ugemm_bf16(std::vector<Variant>& out)
{
    const std::initializer_list<int> sk_all = {1, 2, 4, 8}, sk_few = {1, 2, 4}, sk_one = {1};
    // 16-byte filter loads (C*R*S % 8 == 0)
    ugemm_register<U16CFG(32, 2, 2, 2, 2, 32, true)>(out, sk_few);   // M128 N128
    ugemm_register<U16CFG(32, 2, 2, 2, 1, 32, true)>(out, sk_all);   // M128 N64
    ugemm_register<U16CFG(32, 2, 2, 1, 2, 32, true)>(out, sk_all);   // M64  N128
    ugemm_register<U16CFG(32, 2, 2, 1, 1, 32, true)>(out, sk_all);   // M64  N64
    ugemm_register<U16CFG(32, 1, 4, 1, 1, 32, true)>(out, sk_all);   // M32  N128
    ugemm_register<U16CFG(16, 2, 2, 1, 2, 32, true)>(out, sk_all);   // M32  N64
    ugemm_register<U16CFG(32, 2, 2, 2, 1, 64, true)>(out, sk_few);   // M128 N64
    ugemm_register<U16CFG(32, 2, 2, 2, 2, 64, true)>(out, sk_few);   // M128 N128
    // element-wise filter loads (any C*R*S)
    ugemm_register<U16CFG(32, 1, 4, 3, 1, 32, false)>(out, sk_one);  // M96  N128
    ugemm_register<U16CFG(32, 2, 2, 1, 2, 32, false)>(out, sk_few);  // M64  N128
    ugemm_register<U16CFG(32, 2, 2, 1, 1, 32, false)>(out, sk_few);  // M64  N64
    ugemm_register<U16CFG(32, 1, 4, 1, 1, 32, false)>(out, sk_few);  // M32  N128
    ugemm_register<U16CFG(16, 1, 4, 1, 1, 32, false)>(out, sk_one);  // M16  N64
}

}  // namespace convfwd
