// fp32 instantiations of the scalar-offset implicit-GEMM kernel.
#include "ugemm_kernel.h"

namespace convfwd {

//                 DT        MB WM WN BM BN TK  AVEC
#define U32CFG(MB, WM, WN, BM, BN, TK, AVEC) IgemmCfg<CONV_F32, MB, WM, WN, BM, BN, TK, AVEC, MODE_GATHER>

void register_ugemm_f32(std::vector<Variant>& out)
{
    const std::initializer_list<int> sk_all = {1, 2, 4, 8}, sk_few = {1, 2, 4}, sk_one = {1};
    // 16-byte filter loads
    ugemm_register<U32CFG(32, 2, 2, 2, 2, 16, true)>(out, sk_few);   // M128 N128
    ugemm_register<U32CFG(32, 2, 2, 2, 1, 16, true)>(out, sk_all);   // M128 N64
    ugemm_register<U32CFG(32, 2, 2, 1, 2, 16, true)>(out, sk_all);   // M64  N128
    ugemm_register<U32CFG(32, 2, 2, 1, 1, 16, true)>(out, sk_all);   // M64  N64
    ugemm_register<U32CFG(32, 1, 4, 1, 1, 16, true)>(out, sk_all);   // M32  N128
    ugemm_register<U32CFG(16, 2, 2, 1, 2, 16, true)>(out, sk_all);   // M32  N64
    ugemm_register<U32CFG(32, 1, 4, 3, 1, 16, true)>(out, sk_few);   // M96  N128
    // element-wise filter loads
    ugemm_register<U32CFG(32, 1, 4, 3, 1, 16, false)>(out, sk_one);  // M96  N128
    ugemm_register<U32CFG(32, 2, 2, 1, 2, 16, false)>(out, sk_few);  // M64  N128
    ugemm_register<U32CFG(32, 2, 2, 1, 1, 16, false)>(out, sk_few);  // M64  N64
    ugemm_register<U32CFG(32, 1, 4, 1, 1, 16, false)>(out, sk_few);  // M32  N128
    ugemm_register<U32CFG(16, 1, 4, 1, 1, 16, false)>(out, sk_one);  // M16  N64
    // s-vector gather for unpadded wide windows (first layers)
    ugemm_register_svec<U32CFG(32, 1, 4, 3, 1, 16, true)>(out, sk_one);  // M96  N128
    ugemm_register_svec<U32CFG(32, 2, 2, 1, 2, 16, true)>(out, sk_one);  // M64  N128
    ugemm_register_svec<U32CFG(32, 1, 4, 1, 1, 16, true)>(out, sk_one);  // M32  N128
    ugemm_register_svec<U32CFG(32, 1, 4, 3, 1, 32, true)>(out, sk_one);  // M96  N128 K32
    // twice the reduction step
    ugemm_register<U32CFG(32, 1, 4, 3, 1, 32, false)>(out, sk_one);  // M96  N128
    ugemm_register<U32CFG(32, 1, 4, 3, 1, 32, true)>(out, sk_one);   // M96  N128
    ugemm_register<U32CFG(32, 2, 2, 2, 1, 32, true)>(out, sk_few);   // M128 N64
    ugemm_register<U32CFG(32, 2, 2, 1, 2, 32, true)>(out, sk_few);   // M64  N128
}

}  // namespace convfwd
