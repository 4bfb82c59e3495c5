// fp32 instantiations of the implicit-GEMM kernel (plain fp32 MFMA; gfx950 has no
// reduced-mantissa fp32 MFMA, and the fp32 parity bound would not allow one).
#include "igemm_kernel.h"

namespace convfwd {

//                 DT        MB WM WN BM BN TK  AVEC   MODE
#define F32CFG(MB, WM, WN, BM, BN, AVEC, MODE) IgemmCfg<CONV_F32, MB, WM, WN, BM, BN, 16, AVEC, MODE>
#define F32CFG_K32(MB, WM, WN, BM, BN, AVEC, MODE) IgemmCfg<CONV_F32, MB, WM, WN, BM, BN, 32, AVEC, MODE>

void register_igemm_f32(std::vector<Variant>& out)
{
    const std::initializer_list<int> sk_all = {1, 2, 4, 8}, sk_few = {1, 2, 4}, sk_one = {1};
    // general gather, 16-byte filter loads (needs C*R*S % 4 == 0)
    igemm_register<F32CFG(32, 2, 2, 2, 2, true, MODE_GATHER)>(out, "igemm", FAM_IGEMM, 0, sk_few);   // M128 N128
    igemm_register<F32CFG(32, 2, 2, 2, 1, true, MODE_GATHER)>(out, "igemm", FAM_IGEMM, 0, sk_all);   // M128 N64
    igemm_register<F32CFG(32, 2, 2, 1, 2, true, MODE_GATHER)>(out, "igemm", FAM_IGEMM, 0, sk_all);   // M64  N128
    igemm_register<F32CFG(32, 2, 2, 1, 1, true, MODE_GATHER)>(out, "igemm", FAM_IGEMM, 0, sk_all);   // M64  N64
    igemm_register<F32CFG(32, 1, 4, 1, 1, true, MODE_GATHER)>(out, "igemm", FAM_IGEMM, 0, sk_all);   // M32  N128
    igemm_register<F32CFG(16, 2, 2, 1, 2, true, MODE_GATHER)>(out, "igemm", FAM_IGEMM, 0, sk_all);   // M32  N64
    igemm_register<F32CFG(16, 4, 1, 1, 2, true, MODE_GATHER)>(out, "igemm", FAM_IGEMM, 0, sk_all);   // M64  N32
    // general gather, element-wise filter loads (any C*R*S; first layers)
    igemm_register<F32CFG(32, 2, 2, 2, 2, false, MODE_GATHER)>(out, "igemm", FAM_IGEMM, 0, sk_one);  // M128 N128
    igemm_register<F32CFG(32, 2, 2, 1, 2, false, MODE_GATHER)>(out, "igemm", FAM_IGEMM, 0, sk_few);  // M64  N128
    igemm_register<F32CFG(32, 2, 2, 1, 1, false, MODE_GATHER)>(out, "igemm", FAM_IGEMM, 0, sk_few);  // M64  N64
    igemm_register<F32CFG(32, 1, 4, 3, 1, false, MODE_GATHER)>(out, "igemm", FAM_IGEMM, 0, sk_one);  // M96  N128
    igemm_register<F32CFG(32, 1, 4, 1, 1, false, MODE_GATHER)>(out, "igemm", FAM_IGEMM, 0, sk_few);  // M32  N128
    igemm_register<F32CFG(16, 1, 4, 1, 1, false, MODE_GATHER)>(out, "igemm", FAM_IGEMM, 0, sk_one);  // M16  N64
    igemm_register<F32CFG(16, 2, 2, 1, 2, false, MODE_GATHER)>(out, "igemm", FAM_IGEMM, 0, sk_few);  // M32  N64
    // twice the reduction step: half the barriers and a longer MFMA chain to hide the gather latency behind
    igemm_register<F32CFG_K32(32, 1, 4, 3, 1, false, MODE_GATHER)>(out, "igemm", FAM_IGEMM, 0, sk_one);  // M96  N128
    igemm_register<F32CFG_K32(32, 2, 2, 1, 2, false, MODE_GATHER)>(out, "igemm", FAM_IGEMM, 0, sk_one);  // M64  N128
    igemm_register<F32CFG_K32(32, 2, 2, 2, 1, true, MODE_GATHER)>(out, "igemm", FAM_IGEMM, 0, sk_few);   // M128 N64
    igemm_register<F32CFG_K32(32, 2, 2, 1, 1, true, MODE_GATHER)>(out, "igemm", FAM_IGEMM, 0, sk_few);   // M64  N64
    igemm_register<F32CFG_K32(32, 2, 2, 1, 1, true, MODE_POINTWISE)>(out, "pw", FAM_POINTWISE, 2, sk_few);  // M64 N64
    igemm_register<F32CFG_K32(16, 4, 1, 1, 2, true, MODE_POINTWISE)>(out, "pw", FAM_POINTWISE, 2, sk_few);  // M64 N32
    // pointwise: 1x1, stride 1, pad 0 -- the input image is already the [C x HW] GEMM operand, 16-byte loads along pixels
    igemm_register<F32CFG(32, 2, 2, 2, 1, true, MODE_POINTWISE)>(out, "pw", FAM_POINTWISE, 2, sk_few);  // M128 N64
    igemm_register<F32CFG(32, 2, 2, 1, 2, true, MODE_POINTWISE)>(out, "pw", FAM_POINTWISE, 2, sk_few);  // M64  N128
    igemm_register<F32CFG(32, 2, 2, 1, 1, true, MODE_POINTWISE)>(out, "pw", FAM_POINTWISE, 2, sk_few);  // M64  N64
    igemm_register<F32CFG(32, 1, 4, 1, 1, true, MODE_POINTWISE)>(out, "pw", FAM_POINTWISE, 2, sk_few);  // M32  N128
    igemm_register<F32CFG(16, 2, 2, 1, 2, true, MODE_POINTWISE)>(out, "pw", FAM_POINTWISE, 2, sk_few);  // M32  N64
    igemm_register<F32CFG(16, 4, 1, 1, 2, true, MODE_POINTWISE)>(out, "pw", FAM_POINTWISE, 2, sk_few);  // M64  N32
}

}  // namespace convfwd
