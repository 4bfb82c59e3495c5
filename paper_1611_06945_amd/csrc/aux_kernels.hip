// Second pass of split-reduction variants, and the max-pool helper.
#include <map>
#include <mutex>
#include <utility>

#include <algorithm>
#include <cmath>

#include "igemm_kernel.h"

namespace convfwd {

hipError_t ensure_dynamic_lds(const void* kernel, size_t bytes)
{
    static std::mutex mu;
    static std::map<std::pair<int, const void*>, size_t> raised;  // (device, kernel) -> limit already set
    if (bytes <= 48 * 1024) return hipSuccess;                    // within the default limit
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> g(mu);
    size_t& have = raised[std::make_pair(dev, kernel)];
    if (bytes > have) {
        e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
        if (e != hipSuccess) return e;
        have = bytes;
    }
    return hipSuccess;
}

// out[n,k,pix] = cvt(act(bias[k] + sum_z ws[z][k][p])), z in ascending order so the result does not depend on
// scheduling (no floating-point atomics anywhere).  One thread per output element, pixels fastest.
template <int DT>
__global__ __launch_bounds__(256) void split_reduce_kernel(ConvArgs a)
{
    typedef typename Prec<DT>::elem_t elem_t;
    const size_t total = (size_t)a.K * a.P;
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const uint32_t k = (uint32_t)(i / (size_t)a.P);
    const uint32_t p = (uint32_t)(i - (size_t)k * a.P);
    // the partial sums are fetched eight at a time, all loads in flight before the first addition (a loop of load-then-add
    // would pay one memory latency per split); the additions keep the ascending order
    float x = 0.0f;
    for (int z0 = 0; z0 < a.nsplit; z0 += 8) {
        float v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = (z0 + j < a.nsplit) ? a.ws[(size_t)(z0 + j) * total + i] : 0.0f;
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (z0 + j < a.nsplit) x += v[j];
    }
    if (a.bias) x += a.bias[k];
    if (a.relu) x = x > 0.0f ? x : 0.0f;
    uint32_t n_img, pix;
    a.dOHW.divmod(p, n_img, pix);
    const size_t o = a.out_nhwc ? (size_t)p * a.K + k : ((size_t)n_img * a.K + k) * a.OHW + pix;
    ((elem_t*)a.out)[o] = Prec<DT>::from_f32(x);
}

hipError_t launch_split_reduce(const ConvArgs& a, int dtype, hipStream_t s)
{
    const size_t total = (size_t)a.K * a.P;
    dim3 grid((unsigned)((total + 255) / 256));
    switch (dtype) {
        case CONV_F32: hipLaunchKernelGGL(split_reduce_kernel<CONV_F32>, grid, dim3(256), 0, s, a); break;
        case CONV_F16: hipLaunchKernelGGL(split_reduce_kernel<CONV_F16>, grid, dim3(256), 0, s, a); break;
        default: hipLaunchKernelGGL(split_reduce_kernel<CONV_BF16>, grid, dim3(256), 0, s, a); break;
    }
    return hipGetLastError();
}

// Per-channel max over a win x win window, stride `stride`, no padding.  The 16-bit formats are widened to fp32 for the
// comparison (exact and order preserving) and the winning stored pattern is written back unchanged.  Input and output
// may each be channel-planar ([N][C][H][W]) or channel-innermost ([N][H][W][C]); one thread per output element in the
// order of the output layout, so the pool can double as the layout conversion between two layers.
// WIN = 3: the window is unrolled and its 9 loads are issued together (with a run-time window the loop fetches and
// compares one element at a time, and the kernel's time is 9 memory round trips); WIN = 0: any window, run-time loops.
template <int DT, int WIN>
__global__ __launch_bounds__(256) void maxpool_kernel(const typename Prec<DT>::elem_t* __restrict__ in,
                                                      typename Prec<DT>::elem_t* __restrict__ out, int N, int C, int H, int W,
                                                      int OH, int OW, int win, int stride, int in_nhwc, int out_nhwc,
                                                      FastDiv dOHW, FastDiv dOW, FastDiv dC)
{
    typedef typename Prec<DT>::elem_t elem_t;
    const size_t total = (size_t)N * C * OH * OW;
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    uint32_t n, c, oy, ox;
    if (out_nhwc) {
        uint32_t pix, rem;
        dC.divmod((uint32_t)i, pix, c);
        dOHW.divmod(pix, n, rem);
        dOW.divmod(rem, oy, ox);
    } else {
        uint32_t nc, rem;
        dOHW.divmod((uint32_t)i, nc, rem);
        dOW.divmod(rem, oy, ox);
        dC.divmod(nc, n, c);
    }
    const size_t sy = in_nhwc ? (size_t)W * C : (size_t)W, sx = in_nhwc ? (size_t)C : 1;
    const elem_t* src = in_nhwc ? in + (((size_t)n * H + (size_t)oy * stride) * W + (size_t)ox * stride) * C + c
                                : in + (((size_t)n * C + c) * H + (size_t)oy * stride) * W + (size_t)ox * stride;
    elem_t best = src[0];
    float bestf = Prec<DT>::to_f32(best);
    if constexpr (WIN > 0) {
        elem_t v[WIN * WIN];
#pragma unroll
        for (int r = 0; r < WIN; ++r)
#pragma unroll
            for (int s = 0; s < WIN; ++s) v[r * WIN + s] = src[r * sy + s * sx];
#pragma unroll
        for (int t = 1; t < WIN * WIN; ++t) {
            const float vf = Prec<DT>::to_f32(v[t]);
            if (vf > bestf || vf != vf) {  // a NaN anywhere in the window is the window's result
                bestf = vf;
                best = v[t];
            }
        }
    } else {
        for (int r = 0; r < win; ++r)
            for (int s = 0; s < win; ++s) {
                const elem_t v = src[r * sy + s * sx];
                const float vf = Prec<DT>::to_f32(v);
                if (vf > bestf || vf != vf) {
                    bestf = vf;
                    best = v;
                }
            }
    }
    out[i] = best;
}

// Channel-innermost on both sides with C a multiple of 8: one thread per (output pixel, 8 channels), every tap one
// 16-byte load.  The maximum is taken on the widened values (exact, order preserving) and narrowed back, which is
// exact as well since it is one of the stored values.
template <int DT, int WIN>
__global__ __launch_bounds__(256) void maxpool_nhwc8_kernel(const uint16_t* __restrict__ in, uint16_t* __restrict__ out, int N,
                                                            int C, int H, int W, int OH, int OW, int win, int stride,
                                                            FastDiv dC8, FastDiv dOHW, FastDiv dOW)
{
    const uint32_t total = (uint32_t)N * OH * OW * (C >> 3);
    const uint32_t i = blockIdx.x * 256u + threadIdx.x;
    if (i >= total) return;
    uint32_t pix, oct, n, rem, oy, ox;
    dC8.divmod(i, pix, oct);
    dOHW.divmod(pix, n, rem);
    dOW.divmod(rem, oy, ox);
    const uint16_t* src = in + ((size_t)(n * H + oy * stride) * W + ox * stride) * C + oct * 8;
    float best[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) best[e] = -__builtin_inff();
    auto take = [&](const uint4& v) {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint16_t h = (uint16_t)(e & 1 ? w[e >> 1] >> 16 : w[e >> 1] & 0xFFFFu);
            // the rule of every pooling path: the first of equal values stays (so -0 before +0 stays -0), a NaN sticks
            const float x = Prec<DT>::to_f32(h);
            best[e] = (x > best[e] || x != x) ? x : best[e];
        }
    };
    if constexpr (WIN > 0) {
        uint4 v[WIN * WIN];
#pragma unroll
        for (int r = 0; r < WIN; ++r)
#pragma unroll
            for (int s = 0; s < WIN; ++s) v[r * WIN + s] = *(const uint4*)(src + ((size_t)r * W + s) * C);
#pragma unroll
        for (int t = 0; t < WIN * WIN; ++t) take(v[t]);
    } else {
        for (int r = 0; r < win; ++r)
            for (int s = 0; s < win; ++s) take(*(const uint4*)(src + ((size_t)r * W + s) * C));
    }
    uint32_t o[4];
#pragma unroll
    for (int e = 0; e < 4; ++e)
        o[e] = (uint32_t)Prec<DT>::from_f32(best[2 * e]) | ((uint32_t)Prec<DT>::from_f32(best[2 * e + 1]) << 16);
    *(uint4*)(out + (size_t)i * 8) = make_uint4(o[0], o[1], o[2], o[3]);
}

// The same pooling when input and output layouts differ: a tile of 32 channels x 32 output pixels of one image is
// pooled by threads arranged along the INPUT's contiguous axis, parked in LDS, and written out by threads arranged
// along the OUTPUT's contiguous axis, so that both sides of the conversion move contiguous runs.
template <int DT, bool IN_NHWC, int WIN>
__global__ __launch_bounds__(256) void maxpool_xlayout_kernel(const typename Prec<DT>::elem_t* __restrict__ in,
                                                              typename Prec<DT>::elem_t* __restrict__ out, int C, int H, int W,
                                                              int OH, int OW, int win, int stride, FastDiv dOW)
{
    typedef typename Prec<DT>::elem_t elem_t;
    __shared__ elem_t tile[32][33];  // [channel][pixel]
    const int n = blockIdx.z, c0 = blockIdx.y * 32, p0 = blockIdx.x * 32, OHW = OH * OW;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        // reading side: tx runs along the input's contiguous axis (channels for [N][H][W][C], pixels otherwise)
        const int cl = IN_NHWC ? tx : ty + 8 * j, pl = IN_NHWC ? ty + 8 * j : tx;
        const int c = c0 + cl, p = p0 + pl;
        if (c < C && p < OHW) {
            uint32_t oy, ox;
            dOW.divmod((uint32_t)p, oy, ox);
            const size_t sy = IN_NHWC ? (size_t)W * C : (size_t)W, sx = IN_NHWC ? (size_t)C : 1;
            const elem_t* src = IN_NHWC ? in + (((size_t)n * H + (size_t)oy * stride) * W + (size_t)ox * stride) * C + c
                                        : in + (((size_t)n * C + c) * H + (size_t)oy * stride) * W + (size_t)ox * stride;
            elem_t best = src[0];
            float bestf = Prec<DT>::to_f32(best);
            if constexpr (WIN > 0) {
                elem_t v[WIN * WIN];
#pragma unroll
                for (int r = 0; r < WIN; ++r)
#pragma unroll
                    for (int s = 0; s < WIN; ++s) v[r * WIN + s] = src[r * sy + s * sx];
#pragma unroll
                for (int t = 1; t < WIN * WIN; ++t) {
                    const float vf = Prec<DT>::to_f32(v[t]);
                    if (vf > bestf || vf != vf) {
                        bestf = vf;
                        best = v[t];
                    }
                }
            } else {
                for (int r = 0; r < win; ++r)
                    for (int s = 0; s < win; ++s) {
                        const elem_t v = src[r * sy + s * sx];
                        const float vf = Prec<DT>::to_f32(v);
                        if (vf > bestf || vf != vf) {
                            bestf = vf;
                            best = v;
                        }
                    }
            }
            tile[cl][pl] = best;
        }
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        // writing side: tx runs along the output's contiguous axis (the other one)
        const int cl = IN_NHWC ? ty + 8 * j : tx, pl = IN_NHWC ? tx : ty + 8 * j;
        const int c = c0 + cl, p = p0 + pl;
        if (c < C && p < OHW) {
            if (IN_NHWC)
                out[((size_t)n * C + c) * OHW + p] = tile[cl][pl];
            else
                out[((size_t)n * OHW + p) * C + c] = tile[cl][pl];
        }
    }
}

template <int DT, int WIN>
void launch_maxpool_xlayout(int N, int C, int H, int W, int OH, int OW, int win, int stride, bool in_nhwc, const void* in,
                            void* out, hipStream_t s)
{
    typedef typename Prec<DT>::elem_t elem_t;
    dim3 grid((unsigned)((OH * OW + 31) / 32), (unsigned)((C + 31) / 32), (unsigned)N);
    const FastDiv dOW = make_fastdiv((uint32_t)OW);
    if (in_nhwc)
        hipLaunchKernelGGL((maxpool_xlayout_kernel<DT, true, WIN>), grid, dim3(256), 0, s, (const elem_t*)in, (elem_t*)out, C,
                           H, W, OH, OW, win, stride, dOW);
    else
        hipLaunchKernelGGL((maxpool_xlayout_kernel<DT, false, WIN>), grid, dim3(256), 0, s, (const elem_t*)in, (elem_t*)out, C,
                           H, W, OH, OW, win, stride, dOW);
}

// WIN = 3 (unrolled window) or 0 (any window)
template <int DT, int WIN>
hipError_t launch_maxpool_typed(int N, int C, int H, int W, int win, int stride, bool in_nhwc, bool out_nhwc, const void* in,
                                void* out, hipStream_t s)
{
    typedef typename Prec<DT>::elem_t elem_t;
    const int OH = (H - win) / stride + 1, OW = (W - win) / stride + 1;
    if (in_nhwc != out_nhwc && N <= 65535 && (C + 31) / 32 <= 65535) {
        launch_maxpool_xlayout<DT, WIN>(N, C, H, W, OH, OW, win, stride, in_nhwc, in, out, s);
        return hipGetLastError();
    }
    const size_t total = (size_t)N * C * OH * OW;
    const FastDiv dOHW = make_fastdiv((uint32_t)(OH * OW)), dOW = make_fastdiv((uint32_t)OW), dC = make_fastdiv((uint32_t)C);
    if constexpr (DT != CONV_F32) {
        const bool aligned = ((((uintptr_t)in) | ((uintptr_t)out)) & 15u) == 0;  // its 16-byte loads and stores
        if (in_nhwc && out_nhwc && (C % 8) == 0 && aligned && total / 8 < (1u << 31)) {
            const FastDiv dC8 = make_fastdiv((uint32_t)(C / 8));
            dim3 grid8((unsigned)((total / 8 + 255) / 256));
            hipLaunchKernelGGL((maxpool_nhwc8_kernel<DT, WIN>), grid8, dim3(256), 0, s, (const uint16_t*)in, (uint16_t*)out, N, C,
                               H, W, OH, OW, win, stride, dC8, dOHW, dOW);
            return hipGetLastError();
        }
    }
    dim3 grid((unsigned)((total + 255) / 256));
    hipLaunchKernelGGL((maxpool_kernel<DT, WIN>), grid, dim3(256), 0, s, (const elem_t*)in, (elem_t*)out, N, C, H, W, OH, OW, win,
                       stride, (int)in_nhwc, (int)out_nhwc, dOHW, dOW, dC);
    return hipGetLastError();
}

hipError_t launch_maxpool(int N, int C, int H, int W, int win, int stride, int dtype, bool in_nhwc, bool out_nhwc,
                          const void* in, void* out, hipStream_t s)
{
    const bool w3 = win == 3;
    switch (dtype) {
        case CONV_F32:
            return w3 ? launch_maxpool_typed<CONV_F32, 3>(N, C, H, W, win, stride, in_nhwc, out_nhwc, in, out, s)
                      : launch_maxpool_typed<CONV_F32, 0>(N, C, H, W, win, stride, in_nhwc, out_nhwc, in, out, s);
        case CONV_F16:
            return w3 ? launch_maxpool_typed<CONV_F16, 3>(N, C, H, W, win, stride, in_nhwc, out_nhwc, in, out, s)
                      : launch_maxpool_typed<CONV_F16, 0>(N, C, H, W, win, stride, in_nhwc, out_nhwc, in, out, s);
        default:
            return w3 ? launch_maxpool_typed<CONV_BF16, 3>(N, C, H, W, win, stride, in_nhwc, out_nhwc, in, out, s)
                      : launch_maxpool_typed<CONV_BF16, 0>(N, C, H, W, win, stride, in_nhwc, out_nhwc, in, out, s);
    }
}

// out[a][s][b] = in[a][b][s]: 32x32 tiles through LDS so that both the reads (along s) and the writes (along b) are
// contiguous.  This is the explicit data-format conversion of the paper (Section 3, "Graph-level Optimizations"):
// [N][C][HW] <-> [N][HW][C] for activations and [K][C][RS] -> [K][RS][C] for filters.
template <typename E>
__global__ __launch_bounds__(256) void transpose_kernel(const E* __restrict__ in, E* __restrict__ out, int B, int S)
{
    __shared__ E tile[32][33];
    const int a = blockIdx.z, b0 = blockIdx.y * 32, s0 = blockIdx.x * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
    const E* src = in + (size_t)a * B * S;
    E* dst = out + (size_t)a * B * S;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int b = b0 + ty + 8 * j, s = s0 + tx;
        if (b < B && s < S) tile[ty + 8 * j][tx] = src[(size_t)b * S + s];
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int s = s0 + ty + 8 * j, b = b0 + tx;
        if (b < B && s < S) dst[(size_t)s * B + b] = tile[tx][ty + 8 * j];
    }
}

// Filters [K][C][R][S] -> the MFMA operand order of the packed-filter window kernels:
// out[row block rb][16-channel group c16][tap t][half g][row m][8 channels j] = filt[rb*32 + m][c16*16 + g*8 + j][t],
// zero for rows past K.  One thread writes one 16-byte vector (the 8 channels one lane feeds to a 32x32x16 MFMA).
// This version gathers its 8 values straight from memory: every lane touches another filter row, so it is the fallback
// for windows too large for the LDS version below.
__global__ __launch_bounds__(256) void pack_filters16_kernel(const uint16_t* __restrict__ filt, uint4* __restrict__ out, int K,
                                                            int C, int RS, int nvec)
{
    const int v = blockIdx.x * 256 + threadIdx.x;
    if (v >= nvec) return;
    const int m = v & 31, g = (v >> 5) & 1;
    int rest = v >> 6;
    const int t = rest % RS;
    rest /= RS;
    const int C16 = C >> 4, c16 = rest % C16, rb = rest / C16;
    const int k = rb * 32 + m, c = c16 * 16 + g * 8;
    uint32_t w[4] = {0, 0, 0, 0};
    if (k < K) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t h = filt[((size_t)k * C + c + j) * RS + t];
            w[j >> 1] |= h << ((j & 1) * 16);
        }
    }
    out[v] = make_uint4(w[0], w[1], w[2], w[3]);
}

// The same conversion for one (row block, 16-channel group) per workgroup, through LDS: the 32 rows' pieces (16 channels x
// RS taps, contiguous in [K][C][R][S] and 16-byte aligned because C is a multiple of 16) come in as 16-byte vectors, the
// 8 values of an output vector are gathered from LDS, and consecutive threads write consecutive output vectors.
// `lds` holds 32 rows of 16*RS + 8 elements.
constexpr int kPackMaxRS = 49;  // 7x7: 25 KB of LDS per workgroup
__device__ __forceinline__ void pack_block16(const uint16_t* __restrict__ filt, uint4* __restrict__ out, int K, int C, int RS, int blk,
                                             uint16_t* lds)
{
    const int C16 = C >> 4, rb = blk / C16, c16 = blk - rb * C16;
    const int pitch = 16 * RS + 8, vrow = 2 * RS;  // elements per LDS row; 16-byte vectors per row piece
    for (int v = threadIdx.x; v < 32 * vrow; v += 256) {
        const int row = v / vrow, q = v - row * vrow, k = rb * 32 + row;
        uint4 x = make_uint4(0, 0, 0, 0);
        if (k < K) x = *(const uint4*)(filt + ((size_t)k * C + c16 * 16) * RS + q * 8);
        *(uint4*)&lds[row * pitch + q * 8] = x;
    }
    __syncthreads();
    uint4* dst = out + (size_t)blk * RS * 64;
    for (int v = threadIdx.x; v < 64 * RS; v += 256) {
        const int m = v & 31, g = (v >> 5) & 1, t = v >> 6;
        const uint16_t* src = &lds[m * pitch + g * 8 * RS + t];
        uint32_t w[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) w[j] = (uint32_t)src[2 * j * RS] | ((uint32_t)src[(2 * j + 1) * RS] << 16);
        dst[v] = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

__global__ __launch_bounds__(256) void pack_filters16_lds_kernel(const uint16_t* __restrict__ filt, uint4* __restrict__ out, int K,
                                                                int C, int RS)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t pack_lds[];
    pack_block16(filt, out, K, C, RS, blockIdx.x, pack_lds);
}

// Both conversions a packed-filter kernel needs when it serves a layer handed over in the plain formats, in ONE launch
// ahead of it: blocks [0, in_blocks) transpose the input [N][C][HW] -> [N][HW][C] (32 x 32 tiles through LDS), the
// remaining blocks write the filters in MFMA operand order (one (row block, channel group) each, as above).
__global__ __launch_bounds__(256) void prep16_kernel(const uint16_t* __restrict__ in, uint16_t* __restrict__ in_out, int C, int HW,
                                                    int tiles_s, int tiles_c, int in_blocks, const uint16_t* __restrict__ filt,
                                                    uint4* __restrict__ filt_out, int K, int RS)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t pack_lds[];
    const int b = blockIdx.x;
    if (b < in_blocks) {
        uint16_t(*tile)[33] = (uint16_t(*)[33])pack_lds;  // [32][33]
        const int per_img = tiles_s * tiles_c;
        const int a = b / per_img, rem = b - a * per_img;
        const int b0 = (rem / tiles_s) * 32, s0 = (rem % tiles_s) * 32;
        const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
        const uint16_t* src = in + (size_t)a * C * HW;
        uint16_t* dst = in_out + (size_t)a * C * HW;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = b0 + ty + 8 * j, sidx = s0 + tx;
            if (c < C && sidx < HW) tile[ty + 8 * j][tx] = src[(size_t)c * HW + sidx];
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int sidx = s0 + ty + 8 * j, c = b0 + tx;
            if (c < C && sidx < HW) dst[(size_t)sidx * C + c] = tile[tx][ty + 8 * j];
        }
        return;
    }
    pack_block16(filt, filt_out, K, C, RS, b - in_blocks, pack_lds);
}

static size_t pack_lds_bytes(int RS) { return sizeof(uint16_t) * 32 * (size_t)(16 * RS + 8); }

hipError_t launch_pack_filters16(const void* filt, void* out, int K, int C, int RS, hipStream_t s)
{
    if (RS <= kPackMaxRS) {
        const long long blocks = (long long)((K + 31) / 32) * (C / 16);
        if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
        hipLaunchKernelGGL(pack_filters16_lds_kernel, dim3((unsigned)blocks), dim3(256), pack_lds_bytes(RS), s, (const uint16_t*)filt,
                           (uint4*)out, K, C, RS);
        return hipGetLastError();
    }
    const long long nvec = (long long)((K + 31) / 32) * 32 * (C / 16) * RS * 2;
    hipLaunchKernelGGL(pack_filters16_kernel, dim3((unsigned)((nvec + 255) / 256)), dim3(256), 0, s, (const uint16_t*)filt,
                       (uint4*)out, K, C, RS, (int)nvec);
    return hipGetLastError();
}

// (the packed-filter window kernels exist for 3x3 and 5x5 windows: RS <= kPackMaxRS always holds here)
hipError_t launch_prep16(const void* in, void* in_out, int N, int C, int HW, const void* filt, void* filt_out, int K, int RS,
                         hipStream_t s)
{
    if (RS > kPackMaxRS) return hipErrorInvalidValue;
    const int tiles_s = (HW + 31) / 32, tiles_c = (C + 31) / 32;
    const long long in_blocks = (long long)N * tiles_s * tiles_c;
    const long long blocks = in_blocks + (long long)((K + 31) / 32) * (C / 16);
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const size_t lds = std::max(pack_lds_bytes(RS), sizeof(uint16_t) * 32 * 33);
    hipLaunchKernelGGL(prep16_kernel, dim3((unsigned)blocks), dim3(256), lds, s, (const uint16_t*)in, (uint16_t*)in_out, C, HW,
                       tiles_s, tiles_c, (int)in_blocks, (const uint16_t*)filt, (uint4*)filt_out, K, RS);
    return hipGetLastError();
}

// Reduction behind compare_outputs: stats[0] = bits of max |got - ref|, stats[1] = bits of max |ref| (non-negative floats
// order like their bit patterns), stats[2] = count of elements where got is NaN, or infinite while ref is finite.
template <int DT>
__global__ __launch_bounds__(256) void compare_kernel(const void* got_, const void* ref_, size_t n, uint32_t* stats)
{
    typedef typename Prec<DT>::elem_t elem_t;
    const elem_t* got = (const elem_t*)got_;
    const elem_t* ref = (const elem_t*)ref_;
    float md = 0.0f, mr = 0.0f;
    uint32_t bad = 0;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        const float g = Prec<DT>::to_f32(got[i]), r = Prec<DT>::to_f32(ref[i]);
        const bool rfin = fabsf(r) <= 3.4e38f;
        if (g != g || (!(fabsf(g) <= 3.4e38f) && rfin)) {
            ++bad;
            continue;
        }
        if (!rfin) continue;  // both infinite the same way, or the reference itself overflowed: nothing to compare
        const float d = fabsf(g - r);
        md = d > md ? d : md;
        mr = fabsf(r) > mr ? fabsf(r) : mr;
    }
    __shared__ float smd[256], smr[256];
    __shared__ uint32_t sbad[256];
    smd[threadIdx.x] = md;
    smr[threadIdx.x] = mr;
    sbad[threadIdx.x] = bad;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) {
            smd[threadIdx.x] = fmaxf(smd[threadIdx.x], smd[threadIdx.x + w]);
            smr[threadIdx.x] = fmaxf(smr[threadIdx.x], smr[threadIdx.x + w]);
            sbad[threadIdx.x] += sbad[threadIdx.x + w];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        atomicMax(&stats[0], __builtin_bit_cast(uint32_t, smd[0]));
        atomicMax(&stats[1], __builtin_bit_cast(uint32_t, smr[0]));
        if (sbad[0]) atomicAdd(&stats[2], sbad[0]);
    }
}

hipError_t compare_outputs(int dtype, const void* got, const void* ref, size_t n, uint32_t* stats, hipStream_t s, double* err)
{
    hipError_t e = hipMemsetAsync(stats, 0, 16, s);
    if (e != hipSuccess) return e;
    const unsigned blocks = (unsigned)std::min<size_t>((n + 255) / 256, 2048);
    if (dtype == CONV_F32)
        hipLaunchKernelGGL(compare_kernel<CONV_F32>, dim3(blocks), dim3(256), 0, s, got, ref, n, stats);
    else if (dtype == CONV_F16)
        hipLaunchKernelGGL(compare_kernel<CONV_F16>, dim3(blocks), dim3(256), 0, s, got, ref, n, stats);
    else
        hipLaunchKernelGGL(compare_kernel<CONV_BF16>, dim3(blocks), dim3(256), 0, s, got, ref, n, stats);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    uint32_t h[4] = {0, 0, 0, 0};
    e = hipMemcpyAsync(h, stats, 16, hipMemcpyDeviceToHost, s);
    if (e != hipSuccess) return e;
    e = hipStreamSynchronize(s);
    if (e != hipSuccess) return e;
    const double md = __builtin_bit_cast(float, h[0]), mr = __builtin_bit_cast(float, h[1]);
    *err = h[2] ? (double)INFINITY : md / std::max(mr, 1e-30);
    return hipSuccess;
}

hipError_t launch_transpose(int A, int B, int S, int esize, const void* in, void* out, hipStream_t s)
{
    dim3 grid((unsigned)((S + 31) / 32), (unsigned)((B + 31) / 32), (unsigned)A);
    if (esize == 4)
        hipLaunchKernelGGL(transpose_kernel<uint32_t>, grid, dim3(256), 0, s, (const uint32_t*)in, (uint32_t*)out, B, S);
    else
        hipLaunchKernelGGL(transpose_kernel<uint16_t>, grid, dim3(256), 0, s, (const uint16_t*)in, (uint16_t*)out, B, S);
    return hipGetLastError();
}

}  // namespace convfwd
