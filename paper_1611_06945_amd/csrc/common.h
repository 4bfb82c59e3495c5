// Internal declarations shared by the host dispatcher and the kernel files of
// libconvfwd.so.  Nothing here is part of the public ABI (include/convfwd.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "../../include/convfwd.h"

namespace convfwd {

// Division of a non-negative 31-bit integer by a constant known at launch time.
// The paper's point that ND-Array index arithmetic reduces to chains of constant
// multiplies, divides and modulos (Section 3, "ND-Arrays") is kept: the divisor is
// fixed per launch, so the kernel multiplies and shifts instead of dividing.
//   q = (n * mul) >> shift   exact for 0 <= n < 2^31, 1 <= d < 2^31
// with L = ceil(log2 d), mul = ceil(2^(31+L) / d) (< 2^32), shift = 31 + L.
struct FastDiv {
    uint32_t mul;
    uint32_t shift;
    uint32_t d;
#ifdef __HIPCC__
    __device__ __forceinline__ uint32_t div(uint32_t n) const
    {
        return (uint32_t)(((uint64_t)n * mul) >> shift);
    }
    __device__ __forceinline__ void divmod(uint32_t n, uint32_t& q, uint32_t& r) const
    {
        q = div(n);
        r = n - q * d;
    }
#endif
};

inline FastDiv make_fastdiv(uint32_t d)
{
    FastDiv f;
    uint32_t L = 0;
    while ((1ull << L) < d) ++L;
    uint64_t pw = 1ull << (31 + L);
    f.mul = (uint32_t)((pw + d - 1) / d);
    f.shift = 31 + L;
    f.d = d;
    return f;
}

// Cooperative tile load: `threads` threads fetch `words` words in ceil(words/threads)
// loads each; only the last load needs a guard, and only if words % threads != 0
// (paper, Section 3, "Metaprogramming for NN Convolutions").  constexpr, so the
// kernels unroll their tile loaders from it.
struct CoopPlan {
    int loads;
    bool last_guarded;
};
constexpr CoopPlan coop_plan(int threads, int words)
{
    return CoopPlan{(words + threads - 1) / threads, (words % threads) != 0};
}

// Everything a kernel needs, passed by value.
struct ConvArgs {
    const void* in;
    const void* filt;
    const float* bias;  // may be null
    void* out;
    float* ws;  // partial sums [nsplit][K][P] when nsplit > 1
    int N, C, H, W, K, R, S, stride, pad, OH, OW;
    int P;    // N*OH*OW, the pixel (GEMM-N) extent
    int Q;    // C*R*S, the reduction extent
    int HW;   // H*W
    int OHW;  // OH*OW
    int RS;   // R*S
    int SP4;  // ceil(S/4): 4-column vectors per window row (s-vector gather)
    int QP;   // C*R*4*SP4: reduction extent with window rows padded to a multiple of 4 columns
    int relu;
    int out_nhwc;  // output is [N][OH][OW][K] instead of [N][K][OH][OW]
    int filt_wino; // `filt` already holds the Winograd-domain filters (no transform kernel, no workspace)
    int pool;      // 3x3 stride-2 max-pool fused behind the activation: out is [N][K][POH][POW] (or channel-innermost)
    int POH, POW;  // pooled extent (0 without pool)
    uint32_t in_bytes, filt_bytes, out_bytes;  // extents for the hardware bounds check of tile loads
    int nsplit;           // number of reduction splits (gridDim.z)
    int steps_per_split;  // reduction steps (of the kernel's own step size) per split
    FastDiv dRS, dS, dOHW, dOW, dHW, dW;
    FastDiv dRSP, dSP, dRSP4, dSP4;  // by R*SP, SP = 4*SP4, R*SP4, SP4
    FastDiv dC;                      // by C (channel-innermost reduction axis)
    FastDiv dX, dY, dZ;              // set by the launcher of the kernel family that needs them
};

struct Variant;
typedef hipError_t (*LaunchFn)(const Variant& v, ConvArgs& a, hipStream_t s);
typedef bool (*ValidFn)(const Variant& v, const conv_desc& d, int OH, int OW);
typedef size_t (*WorkspaceFn)(const Variant& v, const conv_desc& d, int OH, int OW);

// One compiled kernel configuration (the paper's "variant + tuning parameters").
struct Variant {
    std::string name;  // e.g. igemm_f32_M128N128K16_w2x2_sk4
    int dtype;         // conv_dtype it is compiled for
    int split;         // reduction splits; 1 = result written directly with the fused epilogue
    int tm, tn, tk;    // workgroup tile: output channels x pixels x reduction step
    int threads;       // workgroup size
    int family;        // FAM_*
    int specificity;   // higher = written for a narrower class of shapes (heuristic tie-break)
    ValidFn valid;
    LaunchFn launch;
    WorkspaceFn ws_extra = nullptr;  // workspace the variant needs beyond split partial sums (null: none)
    unsigned traits = 0;             // TRAIT_* bits read by the cost model used when no measurement exists
};

enum { TRAIT_SCALAR_LOADS = 1u,  // filter tile fetched element by element (no alignment demands, slower steps)
       TRAIT_WHOLE_IMAGE = 2u,   // window kernel whose tile covers complete images
       TRAIT_WINDOW_TILES = 4u,  // tiles are bands of one image's pixels (window-reuse kernels of any family)
       TRAIT_REGISTER_OPERANDS = 8u,  // input operand gathered straight into MFMA registers, no LDS staging of the patch
       TRAIT_STRIDED_VECTOR = 16u,    // gathers four input columns per load on stride-4 layers
       TRAIT_PLANAR_TO_NHWC = 32u,    // reads [N][C][H][W] and [K][C][R][S], can write [N][OH][OW][K] (CONV_FLAG_OUT_NHWC alone)
       TRAIT_FILTERS_IN_KERNEL = 64u,  // Winograd: the filter transform runs inside the product kernel
       TRAIT_POOL_EPILOGUE = 128u,     // can max-pool its output tile before the store (CONV_FLAG_MAXPOOL_3X3S2)
       TRAIT_PACKED_FILTERS = 256u,    // reads filters in MFMA operand order (CONV_FLAG_FILT_PACKED); checks the tensor formats itself
       TRAIT_CONVERTS_FIRST = 512u,    // serves the plain formats by converting input and filters into the workspace first
       TRAIT_WAVE_SPLIT = 1024u,       // the waves of a workgroup split the reduction of one tile (v.threads / 64 ways), operands from global memory
       TRAIT_CHANNEL_WAVES = 2048u };  // fp32 window kernel on linear pixel tiles whose waves split the channels of a chunk

enum { FAM_IGEMM = 0, FAM_POINTWISE = 1, FAM_FIRSTLAYER = 2, FAM_WINDOW = 3, FAM_FC = 4, FAM_NHWC = 5, FAM_WINOGRAD = 6 };

// Each kernel file appends its variants.
void register_igemm_f32(std::vector<Variant>& out);
void register_igemm_f16(std::vector<Variant>& out);
void register_igemm_bf16(std::vector<Variant>& out);
void register_ugemm_f32(std::vector<Variant>& out);
void register_ugemm_f16(std::vector<Variant>& out);
void register_ugemm_bf16(std::vector<Variant>& out);
void register_fc(std::vector<Variant>& out);
void register_nhwc_f16(std::vector<Variant>& out);
void register_nhwc_bf16(std::vector<Variant>& out);
void register_nwin_f16(std::vector<Variant>& out);
void register_nwin_bf16(std::vector<Variant>& out);
void register_swin_f16(std::vector<Variant>& out);
void register_swin_bf16(std::vector<Variant>& out);
void register_swinp_f16(std::vector<Variant>& out);
void register_swinp_bf16(std::vector<Variant>& out);
void register_wconv_f32(std::vector<Variant>& out);
void register_wconv_f16(std::vector<Variant>& out);
void register_wconv_bf16(std::vector<Variant>& out);
void register_wino_f32(std::vector<Variant>& out);
void register_pwk_f32(std::vector<Variant>& out);
void register_pwk_f16(std::vector<Variant>& out);
void register_pwk_bf16(std::vector<Variant>& out);
void register_pwin32_f32(std::vector<Variant>& out);
void register_pwin_f16(std::vector<Variant>& out);
void register_pwin_bf16(std::vector<Variant>& out);

// Raises a kernel's dynamic-LDS limit to `bytes` on the current device when it is not already that high (once per
// device and kernel; safe to call from several threads).
hipError_t ensure_dynamic_lds(const void* kernel, size_t bytes);

// Split-reduction second pass and the max-pool helper (aux_kernels.hip).
hipError_t launch_split_reduce(const ConvArgs& a, int dtype, hipStream_t s);
hipError_t launch_maxpool(int N, int C, int H, int W, int win, int stride, int dtype, bool in_nhwc, bool out_nhwc,
                          const void* in, void* out, hipStream_t s);
// out[a][s][b] = in[a][b][s] for elements of `esize` bytes (2 or 4): the layout conversions of tensors and filters
hipError_t launch_transpose(int A, int B, int S, int esize, const void* in, void* out, hipStream_t s);
// Winograd filter transform in the layout of the 8-channel-step variants (wino_f32.hip); bytes = 16 * K' * C * 4
hipError_t launch_wino_filter_transform(const float* filt, float* out, int K, int C, hipStream_t s);
size_t wino_transformed_filter_bytes(int K, int C);
// KCRS 16-bit filters -> MFMA operand order of the packed-filter kernels (aux_kernels.hip); C % 16 == 0
// input [N][C][HW] -> [N][HW][C] and filters -> MFMA operand order in one launch (aux_kernels.hip); C % 16 == 0
hipError_t launch_prep16(const void* in, void* in_out, int N, int C, int HW, const void* filt, void* filt_out, int K, int RS,
                         hipStream_t s);
hipError_t launch_pack_filters16(const void* filt, void* out, int K, int C, int RS, hipStream_t s);

// max_i |got_i - ref_i| / max(max_j |ref_j|, 1e-30) of two device tensors of `n` elements (infinity when `got` holds a
// non-finite value where `ref` is finite, or a NaN); `stats` is 16 bytes of device scratch.  Synchronises `s`.
hipError_t compare_outputs(int dtype, const void* got, const void* ref, size_t n, uint32_t* stats, hipStream_t s, double* err);

// Device ceilings measured in place (probe_kernels.hip).
hipError_t probe_mfma(int dtype, int block, float* sink, hipStream_t s, double* tflops);
hipError_t probe_mfma_mix(int dtype, int block, int wps, int nv, int distinct, float* sink, hipStream_t s, double* tflops, double* ns);
hipError_t probe_copy(const void* src, void* dst, size_t bytes, hipStream_t s, double* gbs);

inline const char* dtype_name(int dt) { return dt == CONV_F32 ? "f32" : dt == CONV_F16 ? "f16" : "bf16"; }
inline int dtype_size(int dt) { return dt == CONV_F32 ? 4 : 2; }

}  // namespace convfwd
