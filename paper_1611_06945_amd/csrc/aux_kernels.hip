// Second pass of split-reduction variants, and the max-pool helper.
#include "igemm_kernel.h"

namespace convfwd {

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
    float x = 0.0f;
    for (int z = 0; z < a.nsplit; ++z) x += a.ws[(size_t)z * total + i];
    if (a.bias) x += a.bias[k];
    if (a.relu) x = x > 0.0f ? x : 0.0f;
    uint32_t n_img, pix;
    a.dOHW.divmod(p, n_img, pix);
    ((elem_t*)a.out)[((size_t)n_img * a.K + k) * a.OHW + pix] = Prec<DT>::from_f32(x);
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
// comparison (exact and order preserving) and the winning stored pattern is written back unchanged.
template <int DT>
__global__ __launch_bounds__(256) void maxpool_kernel(const typename Prec<DT>::elem_t* __restrict__ in,
                                                      typename Prec<DT>::elem_t* __restrict__ out, int NC, int H, int W,
                                                      int OH, int OW, int win, int stride, FastDiv dOHW, FastDiv dOW)
{
    typedef typename Prec<DT>::elem_t elem_t;
    const size_t total = (size_t)NC * OH * OW;
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    uint32_t nc, rem, oy, ox;
    dOHW.divmod((uint32_t)i, nc, rem);
    dOW.divmod(rem, oy, ox);
    const elem_t* src = in + ((size_t)nc * H + (size_t)oy * stride) * W + (size_t)ox * stride;
    elem_t best = src[0];
    float bestf = Prec<DT>::to_f32(best);
    for (int r = 0; r < win; ++r)
        for (int s = 0; s < win; ++s) {
            const elem_t v = src[(size_t)r * W + s];
            const float vf = Prec<DT>::to_f32(v);
            if (vf > bestf) {
                bestf = vf;
                best = v;
            }
        }
    out[i] = best;
}

hipError_t launch_maxpool(int N, int C, int H, int W, int win, int stride, int dtype, const void* in, void* out,
                          hipStream_t s)
{
    const int OH = (H - win) / stride + 1, OW = (W - win) / stride + 1;
    const size_t total = (size_t)N * C * OH * OW;
    dim3 grid((unsigned)((total + 255) / 256));
    const FastDiv dOHW = make_fastdiv((uint32_t)(OH * OW)), dOW = make_fastdiv((uint32_t)OW);
    switch (dtype) {
        case CONV_F32:
            hipLaunchKernelGGL(maxpool_kernel<CONV_F32>, grid, dim3(256), 0, s, (const float*)in, (float*)out, N * C, H,
                               W, OH, OW, win, stride, dOHW, dOW);
            break;
        case CONV_F16:
            hipLaunchKernelGGL(maxpool_kernel<CONV_F16>, grid, dim3(256), 0, s, (const uint16_t*)in, (uint16_t*)out,
                               N * C, H, W, OH, OW, win, stride, dOHW, dOW);
            break;
        default:
            hipLaunchKernelGGL(maxpool_kernel<CONV_BF16>, grid, dim3(256), 0, s, (const uint16_t*)in, (uint16_t*)out,
                               N * C, H, W, OH, OW, win, stride, dOHW, dOW);
            break;
    }
    return hipGetLastError();
}

}  // namespace convfwd
