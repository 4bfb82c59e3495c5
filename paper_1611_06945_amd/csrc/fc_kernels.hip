// Fully-connected layers written as convolutions: the window covers the whole input (R == H, S == W, no padding), so
// there is one output pixel per image and
//     out[n][k] = act(bias[k] + sum_q filt[k][q] * in[n][q]),   q = (c, r, s) = the NCHW order of image n.
// The paper lists these layers in its benchmark set (Appendix A: 6x6x256 -> 4096 and 1x1x4096 -> 4096 at batch 5) and
// names them as the outlier its convolution variants do not handle well (Section 4, "Experimental Results").  With a
// handful of images every weight is used only N times: the layer streams the filter tensor once from HBM and is bound
// by that stream, not by arithmetic -- so this kernel is a plain vector-ALU dot product organised around the loads:
//   * a workgroup owns ROWS output channels; its four waves split the reduction axis, every lane walks it with
//     16-byte loads (a wave reads 1 KiB of one filter row per instruction);
//   * the input vectors are read with the same pattern from L2 and reused for all ROWS rows in registers, which keeps
//     the load traffic at (1 + N/ROWS) times the filter bytes;
//   * partial sums are added lane by lane (fixed butterfly order), then wave by wave through LDS: deterministic.
#include "igemm_kernel.h"

namespace convfwd {

namespace {

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// acc += dot(w, x) over the VEC elements of one 16-byte vector of each operand, accumulated in fp32.  16-bit pairs go
// through the two-element dot instructions (exact products, fp32 sum), which halves the vector-ALU work per byte.
template <int DT>
struct FcVec;
template <>
struct FcVec<CONV_F32> {
    static constexpr int VEC = 4;
    static __device__ __forceinline__ float mac(const uint4& w, const uint4& x, float acc)
    {
        acc = __builtin_fmaf(__builtin_bit_cast(float, w.x), __builtin_bit_cast(float, x.x), acc);
        acc = __builtin_fmaf(__builtin_bit_cast(float, w.y), __builtin_bit_cast(float, x.y), acc);
        acc = __builtin_fmaf(__builtin_bit_cast(float, w.z), __builtin_bit_cast(float, x.z), acc);
        acc = __builtin_fmaf(__builtin_bit_cast(float, w.w), __builtin_bit_cast(float, x.w), acc);
        return acc;
    }
};
template <>
struct FcVec<CONV_F16> {
    static constexpr int VEC = 8;
    static __device__ __forceinline__ float mac(const uint4& w, const uint4& x, float acc)
    {
        acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, w.x), __builtin_bit_cast(f16x2, x.x), acc, false);
        acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, w.y), __builtin_bit_cast(f16x2, x.y), acc, false);
        acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, w.z), __builtin_bit_cast(f16x2, x.z), acc, false);
        acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, w.w), __builtin_bit_cast(f16x2, x.w), acc, false);
        return acc;
    }
};
template <>
struct FcVec<CONV_BF16> {
    static constexpr int VEC = 8;
    static __device__ __forceinline__ float mac(const uint4& w, const uint4& x, float acc)
    {
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w.x), __builtin_bit_cast(bf16x2, x.x), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w.y), __builtin_bit_cast(bf16x2, x.y), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w.z), __builtin_bit_cast(bf16x2, x.z), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w.w), __builtin_bit_cast(bf16x2, x.w), acc, false);
        return acc;
    }
};

constexpr int kFcThreads = 256;  // four waves

template <int DT, int ROWS, int NB>
__global__ __launch_bounds__(kFcThreads) void fc_kernel(ConvArgs a)
{
    typedef typename Prec<DT>::elem_t elem_t;
    constexpr int VEC = FcVec<DT>::VEC;
    constexpr uint32_t ES = sizeof(elem_t);
    __shared__ float red[4][ROWS][NB];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int k0 = blockIdx.x * ROWS;
    const __amdgpu_buffer_rsrc_t rin = make_rsrc(a.in, a.in_bytes);
    const __amdgpu_buffer_rsrc_t rfilt = make_rsrc(a.filt, a.filt_bytes);

    float acc[ROWS][NB];
#pragma unroll
    for (int r = 0; r < ROWS; ++r)
#pragma unroll
        for (int n = 0; n < NB; ++n) acc[r][n] = 0.0f;

    // byte offsets of this workgroup's filter rows and of the images (rows past K / images past N read as zero)
    uint32_t row_off[ROWS], img_off[NB];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) row_off[r] = (k0 + r < a.K) ? (uint32_t)(k0 + r) * (uint32_t)a.Q * ES : kOutOfRange;
#pragma unroll
    for (int n = 0; n < NB; ++n) img_off[n] = (n < a.N) ? (uint32_t)n * (uint32_t)a.Q * ES : kOutOfRange;

    // the reduction axis in vectors: wave w takes vectors w*64 + lane, + 256, + 512, ...
    const int nvec = a.Q / VEC;
#pragma unroll 2
    for (int v = tid; v < nvec; v += kFcThreads) {
        const uint32_t col = (uint32_t)v * (uint32_t)(VEC * ES);
        uint4 wv[ROWS], xv[NB];
#pragma unroll
        for (int r = 0; r < ROWS; ++r) wv[r] = buffer_load_vec(rfilt, row_off[r] == kOutOfRange ? kOutOfRange : row_off[r] + col);
#pragma unroll
        for (int n = 0; n < NB; ++n) xv[n] = buffer_load_vec(rin, img_off[n] == kOutOfRange ? kOutOfRange : img_off[n] + col);
#pragma unroll
        for (int r = 0; r < ROWS; ++r)
#pragma unroll
            for (int n = 0; n < NB; ++n) acc[r][n] = FcVec<DT>::mac(wv[r], xv[n], acc[r][n]);
    }

    // lanes of a wave: butterfly over lane distance 32, 16, ..., 1 (the same order in every launch)
#pragma unroll
    for (int r = 0; r < ROWS; ++r)
#pragma unroll
        for (int n = 0; n < NB; ++n) {
            float x = acc[r][n];
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d, 64);
            acc[r][n] = x;
        }
    if (lane == 0) {
#pragma unroll
        for (int r = 0; r < ROWS; ++r)
#pragma unroll
            for (int n = 0; n < NB; ++n) red[wave][r][n] = acc[r][n];
    }
    __syncthreads();
    if (tid < ROWS * NB) {
        const int r = tid / NB, n = tid % NB;
        const int k = k0 + r;
        if (k < a.K && n < a.N) {
            float x = ((red[0][r][n] + red[1][r][n]) + red[2][r][n]) + red[3][r][n];
            if (a.bias) x += a.bias[k];
            if (a.relu & 1) x = x > 0.0f ? x : 0.0f;
            ((elem_t*)a.out)[(size_t)n * a.K + k] = Prec<DT>::from_f32(x);
        }
    }
}

template <int DT, int ROWS, int NB>
hipError_t fc_launch(const Variant& v, ConvArgs& a, hipStream_t s)
{
    a.nsplit = 1;
    a.steps_per_split = 0;
    dim3 grid((unsigned)((a.K + ROWS - 1) / ROWS));
    hipLaunchKernelGGL((fc_kernel<DT, ROWS, NB>), grid, dim3(kFcThreads), 0, s, a);
    return hipGetLastError();
}

template <int DT, int ROWS, int NB, int NB_BELOW>
bool fc_valid(const Variant& v, const conv_desc& d, int OH, int OW)
{
    if (d.dtype != DT) return false;
    if (OH != 1 || OW != 1 || d.pad != 0 || d.R != d.H || d.S != d.W) return false;  // the window is the whole image
    const long long Q = (long long)d.C * d.R * d.S;
    if (Q % FcVec<DT>::VEC != 0) return false;              // rows and images start on 16-byte boundaries
    if (d.N > NB || d.N <= NB_BELOW) return false;  // one pass over the weights, in the smallest instantiation that holds N
    if ((long long)d.K > 2147483647LL * ROWS / 2) return false;
    return true;
}

template <int DT, int ROWS, int NB, int NB_BELOW>
void fc_register_one(std::vector<Variant>& out)
{
    Variant v;
    char buf[96];
    snprintf(buf, sizeof buf, "fc_%s_rows%d_n%d", dtype_name(DT), ROWS, NB);
    v.name = buf;
    v.dtype = DT;
    v.split = 1;
    v.tm = ROWS;
    v.tn = NB;
    v.tk = 256 * FcVec<DT>::VEC;
    v.threads = kFcThreads;
    v.family = FAM_FC;
    v.specificity = 6;
    v.valid = &fc_valid<DT, ROWS, NB, NB_BELOW>;
    v.launch = &fc_launch<DT, ROWS, NB>;
    out.push_back(v);
}

// image counts 1, 2, 3-4, 5, 6, 7-8 (5 is the paper's batch); NB_BELOW = the next smaller instantiation
template <int DT, int ROWS>
void fc_register_rows(std::vector<Variant>& out)
{
    fc_register_one<DT, ROWS, 1, 0>(out);
    fc_register_one<DT, ROWS, 2, 1>(out);
    fc_register_one<DT, ROWS, 4, 2>(out);
    fc_register_one<DT, ROWS, 5, 4>(out);
    fc_register_one<DT, ROWS, 6, 5>(out);
    fc_register_one<DT, ROWS, 8, 6>(out);
}
template <int DT>
void fc_register_dtype(std::vector<Variant>& out)
{
    fc_register_rows<DT, 2>(out);
    fc_register_rows<DT, 4>(out);
    fc_register_rows<DT, 8>(out);
}

}  // namespace

void register_fc(std::vector<Variant>& out)
{
    fc_register_dtype<CONV_F32>(out);
    fc_register_dtype<CONV_F16>(out);
    fc_register_dtype<CONV_BF16>(out);
}

}  // namespace convfwd
