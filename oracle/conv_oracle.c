/*
 * CPU oracle for forward 2D convolution with fused bias + ReLU, and for the
 * spatial max-pool that sits between layers of a convolution stack.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing on the product path may call, link or load
 * this file; it exists so that the GPU library has an independent, slow and
 * obviously correct result to be compared with.  It shares no source, header,
 * table or helper with the HIP library.
 *
 * What it computes (paper, Section 2 "Background", the paragraph that defines a
 * convolution layer as output = conv(input, filters): every output value is the
 * dot product of one filter's weights with a window of the input, the window
 * being slid over the input with a spatial stride; Appendix A: square or
 * rectangular windows, one stride for both spatial axes; Section 3
 * "Graph-level Optimizations": the activation that follows the convolution is
 * applied on each output write):
 *
 *   out[n,k,oy,ox] = act( bias[k] + sum_{c,r,s} in[n,c,oy*stride-pad+r,
 *                                                   ox*stride-pad+s] * filt[k,c,r,s] )
 *
 * with terms whose input coordinate falls outside [0,H) x [0,W) contributing
 * zero (zero padding), OH = floor((H+2*pad-R)/stride)+1 and OW likewise (floor
 * is what reproduces every "in -> out" size pair of the Appendix A table), no
 * filter flip (cross-correlation), act = max(x,0) when relu != 0, else identity.
 *
 * Everything is fp64: inputs are handed over as doubles (the caller widens the
 * stored fp32 / fp16 / bf16 values exactly), the accumulator is a double, the
 * result is left in double and is never rounded to a storage type.  Loops are
 * the definition written out: no tiling, no blocking, no reordering.  OpenMP
 * splits the (n,k) pairs over threads only to bound wall time; each output is
 * still accumulated by one thread in the fixed order c, r, s.
 *
 * Layouts: in [N][C][H][W], filt [K][C][R][S], bias [K] (or NULL),
 * out [N][K][OH][OW]; all dense, C order.
 *
 * Pins (tests/test_oracle_pins.py): pure-Python brute force on tiny shapes,
 * identity and shifted-delta filters, 1x1 == matrix product, full-size filter
 * == dot product, linearity, all-ones closed form under padding and stride,
 * zero input -> act(bias), and the output sizes of Appendix A.
 */
#include <stddef.h>
#include <stdint.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* Output extent along one axis; returns 0 when the window does not fit. */
static int64_t out_extent(int64_t in_sz, int64_t win, int64_t stride, int64_t pad)
{
    int64_t span = in_sz + 2 * pad - win;
    if (span < 0) return 0;
    return span / stride + 1; /* span >= 0, so C division is floor */
}

int oracle_conv_out_shape(int H, int W, int R, int S, int stride, int pad, int *OH, int *OW)
{
    if (H < 1 || W < 1 || R < 1 || S < 1 || stride < 1 || pad < 0) return -1;
    int64_t oh = out_extent(H, R, stride, pad);
    int64_t ow = out_extent(W, S, stride, pad);
    if (oh < 1 || ow < 1) return -1;
    *OH = (int)oh;
    *OW = (int)ow;
    return 0;
}

/* One output value, straight from the definition. */
static double conv_point(int C, int H, int W, int R, int S, int stride, int pad,
                         const double *in_n, /* [C][H][W] of image n */
                         const double *filt_k, /* [C][R][S] of filter k */
                         const double *bias, int k, int relu, int oy, int ox)
{
    double acc = 0.0;
    for (int c = 0; c < C; ++c) {
        for (int r = 0; r < R; ++r) {
            int iy = oy * stride - pad + r;
            if (iy < 0 || iy >= H) continue;
            for (int s = 0; s < S; ++s) {
                int ix = ox * stride - pad + s;
                if (ix < 0 || ix >= W) continue;
                acc += in_n[((size_t)c * H + iy) * W + ix] * filt_k[((size_t)c * R + r) * S + s];
            }
        }
    }
    if (bias) acc += bias[k];
    if (relu && !(acc > 0.0)) acc = 0.0;
    return acc;
}

int oracle_conv_fwd(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                    const double *in, const double *filt, const double *bias, int relu,
                    double *out)
{
    int OH, OW;
    if (N < 1 || C < 1 || K < 1 || !in || !filt || !out) return -1;
    if (oracle_conv_out_shape(H, W, R, S, stride, pad, &OH, &OW)) return -1;
    const size_t in_img = (size_t)C * H * W, filt_one = (size_t)C * R * S;
    const size_t out_plane = (size_t)OH * OW;
    const long NK = (long)N * K;
#pragma omp parallel for schedule(static)
    for (long nk = 0; nk < NK; ++nk) {
        int n = (int)(nk / K), k = (int)(nk % K);
        double *o = out + ((size_t)n * K + k) * out_plane;
        for (int oy = 0; oy < OH; ++oy)
            for (int ox = 0; ox < OW; ++ox)
                o[(size_t)oy * OW + ox] = conv_point(C, H, W, R, S, stride, pad, in + n * in_img,
                                                     filt + k * filt_one, bias, k, relu, oy, ox);
    }
    return 0;
}

/*
 * The same definition evaluated only at chosen outputs: idx[i] is a flat index
 * into out[N][K][OH][OW]; vals[i] receives that output.  Used at sizes where the
 * whole output would take the CPU too long.
 */
int oracle_conv_fwd_points(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                           const double *in, const double *filt, const double *bias, int relu,
                           long n_points, const int64_t *idx, double *vals)
{
    int OH, OW;
    if (N < 1 || C < 1 || K < 1 || !in || !filt || !idx || !vals || n_points < 0) return -1;
    if (oracle_conv_out_shape(H, W, R, S, stride, pad, &OH, &OW)) return -1;
    const size_t in_img = (size_t)C * H * W, filt_one = (size_t)C * R * S;
    const int64_t total = (int64_t)N * K * OH * OW;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (long i = 0; i < n_points; ++i) {
        int64_t f = idx[i];
        if (f < 0 || f >= total) {
            bad = 1;
            continue;
        }
        int ox = (int)(f % OW);
        f /= OW;
        int oy = (int)(f % OH);
        f /= OH;
        int k = (int)(f % K);
        int n = (int)(f / K);
        vals[i] = conv_point(C, H, W, R, S, stride, pad, in + n * in_img, filt + k * filt_one, bias,
                             k, relu, oy, ox);
    }
    return bad ? -1 : 0;
}

/*
 * Spatial max-pool, per channel, window win x win, stride `stride`, no padding,
 * output extent floor((H-win)/stride)+1 (paper, Section 2: pooling works per
 * channel over a small window, about win*win comparisons per output pixel).
 * in [N][C][H][W] -> out [N][C][OH][OW].
 */
int oracle_maxpool_fwd(int N, int C, int H, int W, int win, int stride, const double *in,
                       double *out)
{
    if (N < 1 || C < 1 || win < 1 || stride < 1 || H < win || W < win || !in || !out) return -1;
    const int OH = (H - win) / stride + 1, OW = (W - win) / stride + 1;
    const long NC = (long)N * C;
#pragma omp parallel for schedule(static)
    for (long nc = 0; nc < NC; ++nc) {
        const double *src = in + (size_t)nc * H * W;
        double *dst = out + (size_t)nc * OH * OW;
        for (int oy = 0; oy < OH; ++oy)
            for (int ox = 0; ox < OW; ++ox) {
                double m = src[(size_t)(oy * stride) * W + ox * stride];
                for (int r = 0; r < win; ++r)
                    for (int s = 0; s < win; ++s) {
                        double v = src[(size_t)(oy * stride + r) * W + ox * stride + s];
                        if (v > m) m = v;
                    }
                dst[(size_t)oy * OW + ox] = m;
            }
    }
    return 0;
}

/* Threads the parallel loops above will use (1 when built without OpenMP). */
int oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
