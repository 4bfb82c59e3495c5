// Window-reuse convolution for stride-1 layers, fp16 / bf16 storage (32x32x16 MFMA, fp32 accumulate).
//
// Same idea as the fp32 window kernel (the input is copied once into LDS and every tap of the window is an LDS
// read at a constant offset, so overlapping windows share the copy; paper, Section 5 "Related Work": what
// im2col + GEMM forfeits), re-laid for the 16-bit MFMA operand shape, where a lane feeds 8 consecutive reduction
// elements per instruction:
//   * workgroup = TM output channels x one band of BH output rows of one image (BH*OW <= TNP pixel columns);
//   * chunk = CB = 16*KW input channels.  The band's input rows go to LDS channel-innermost, [position][channel]
//     with a zero border, so a lane's patch operand for tap (r,s) is ONE 16-byte LDS read of 8 consecutive
//     channels at position pixel + r*PW + s.  The transposition from NCHW happens once per chunk while staging
//     (eight 2-byte loads of one pixel across eight channels -> one 16-byte LDS write);
//   * the filter slab keeps its KCRS order, [TM][CB*R*S] (16-byte copies); a lane's filter operand is the same 8
//     channels at one tap: the lane reads its 8*R*S consecutive filter elements once per chunk (16-byte LDS reads)
//     and assembles each tap's operand in registers with byte permutes;
//   * KW waves split the chunk's channels (16 each), WN waves split the pixel blocks; partial sums of the KW
//     channel-waves are added in wave order through LDS (deterministic), then bias + activation + rounding + store.
#pragma once

#include <type_traits>

#include "igemm_kernel.h"

namespace convfwd {

template <int DT_, int R_, int S_, int KW_, int WM_, int TMB_, int WN_, int NBW_, int LBT_, int LBN_ = 0>
struct Wconv16Cfg {
    static_assert(DT_ == CONV_F16 || DT_ == CONV_BF16, "16-bit storage only");
    static constexpr int DT = DT_, R = R_, S = S_, KW = KW_, WM = WM_, TMB = TMB_, WN = WN_, NBW = NBW_, LBT = LBT_;
    // LBN > 0: the band is the whole image and its [CB][H*W] slab, contiguous and 16-byte aligned in global memory, is
    // copied with LBN 16-byte loads per thread into a plain LDS buffer first and transposed from there (LDS to LDS);
    // LBN = 0: the slab is gathered with 2-byte loads (any band, any alignment).
    static constexpr int LBN = LBN_;
    static constexpr int RS = R * S;
    static constexpr int NT = 64 * KW * WM * WN;
    static constexpr int CB = 16 * KW;                 // channels per chunk
    static constexpr int TM = 32 * TMB * WM;           // output channels per workgroup
    static constexpr int TNP = 32 * NBW * WN;          // pixel columns per workgroup
    static constexpr int KCH = CB * RS;                // reduction elements per chunk
    static constexpr int LDA = KCH + 8;                // filter slab row pitch (16-bit elements), keeps rows 16-byte aligned
    static constexpr int CP = CB + 8;                  // channel pitch of one LDS position
    static constexpr CoopPlan planA = coop_plan(NT, TM * KCH / 8);
    static constexpr int RED_FLOATS = KW * 32 * TNP;   // reduction buffer, one 32-row block at a time
};

struct Wconv16Geom {
    int band_h;    // output rows per workgroup
    int bands;     // workgroups per image
    int in_rows;   // input rows one band touches, border included: band_h + R - 1
    int npos;      // LDS positions of one band: in_rows * PW, plus slack for lanes without a pixel
};

template <class CFG>
__host__ __device__ inline Wconv16Geom wconv16_geom(int W, int pad, int OH, int OW)
{
    Wconv16Geom g;
    g.band_h = CFG::TNP / OW;
    if (g.band_h > OH) g.band_h = OH;
    if (g.band_h < 1) g.band_h = 1;
    g.bands = (OH + g.band_h - 1) / g.band_h;
    g.in_rows = g.band_h + CFG::R - 1;
    g.npos = g.in_rows * (W + 2 * pad) + 8;
    return g;
}

template <class CFG>
__global__ __launch_bounds__(CFG::NT) void wconv16_kernel(ConvArgs a)
{
    typedef uint16_t elem_t;
    constexpr int DT = CFG::DT, R = CFG::R, S = CFG::S, RS = CFG::RS, KW = CFG::KW, WM = CFG::WM, TMB = CFG::TMB;
    constexpr int WN = CFG::WN, NBW = CFG::NBW, LBT = CFG::LBT, NT = CFG::NT, CB = CFG::CB, TM = CFG::TM, TNP = CFG::TNP;
    constexpr int KCH = CFG::KCH, LDA = CFG::LDA, CP = CFG::CP, LBN = CFG::LBN;
    constexpr bool NAT = LBN > 0;
    constexpr CoopPlan planA = CFG::planA;
    typedef Mma<DT, 32> mma_t;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];

    const Wconv16Geom geo = wconv16_geom<CFG>(a.W, a.pad, a.OH, a.OW);
    const int PW = a.W + 2 * a.pad;
    elem_t* const As0 = (elem_t*)smem_raw;              // [2][TM*LDA]
    elem_t* const Bs0 = As0 + 2 * TM * LDA;             // [2][npos*CP]
    const int b_elems = geo.npos * CP;
    elem_t* const Nat = Bs0 + 2 * b_elems;               // [CB][H*W] raw copy of the chunk's image slab (LBN > 0 only)

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int kw = wave % KW, wn = (wave / KW) % WN, wm = wave / (KW * WN);
    const int li = lane & 31, g = lane >> 5;

    const int img = blockIdx.x / geo.bands, band = blockIdx.x - img * geo.bands;
    const int oy0 = band * geo.band_h;
    const int bh = (a.OH - oy0 < geo.band_h) ? a.OH - oy0 : geo.band_h;  // output rows of this band
    const int npix = bh * a.OW;                                          // real pixel columns of this band
    const int m0 = blockIdx.y * TM;

    const int total_chunks = a.C / CB;
    const int chunk_begin = blockIdx.z * a.steps_per_split;
    int chunk_end = chunk_begin + a.steps_per_split;
    if (chunk_end > total_chunks) chunk_end = total_chunks;

    const __amdgpu_buffer_rsrc_t rin = make_rsrc(a.in, a.in_bytes);
    const __amdgpu_buffer_rsrc_t rfilt = make_rsrc(a.filt, a.filt_bytes);

    // ---- staging plan of the patch slab: task = (input pixel of the band, channel octet) -----------------------
    // input rows iy in [iy_lo, iy_hi) of the image are the band's rows oy0-pad .. oy0-pad+in_rows-1 clipped to the image
    const int iy_first = oy0 - a.pad;
    const int iy_lo = iy_first < 0 ? 0 : iy_first;
    int iy_hi = iy_first + bh + R - 1;
    if (iy_hi > a.H) iy_hi = a.H;
    const int band_pix = (iy_hi - iy_lo) * a.W;           // contiguous in global memory for one channel
    const int ntask = band_pix * (CB / 8);
    int t_goff[LBT];   // element offset of (channel octet's first channel, pixel) relative to the chunk's first channel
    int t_lds[LBT];    // element index in the LDS slab, or -1
    int t_nat[LBT];    // element index of (octet's first channel, pixel) in the raw LDS copy (LBN > 0)
#pragma unroll
    for (int i = 0; i < LBT; ++i) {
        const int t = i * NT + tid;
        const bool ok = t < ntask;
        const int oct = ok ? t / band_pix : 0;
        const int pix = ok ? t - oct * band_pix : 0;
        uint32_t y, x;
        a.dW.divmod((uint32_t)pix, y, x);
        t_goff[i] = (oct * 8) * a.HW + iy_lo * a.W + pix;
        t_nat[i] = t_goff[i];
        t_lds[i] = ok ? ((iy_lo - iy_first + (int)y) * PW + (int)x + a.pad) * CP + oct * 8 : -1;
    }

    uint4 a_reg[planA.loads];
    elem_t b_reg[NAT ? 1 : LBT][8];
    uint4 n_reg[NAT ? LBN : 1];
    const int nvecN = (CB * a.HW) >> 3;  // 16-byte vectors of one [CB][H*W] slab

    auto load_chunk = [&](int chunk) {
        const int c0 = chunk * CB;
#pragma unroll
        for (int i = 0; i < planA.loads; ++i) {
            const int v = i * NT + tid;
            const bool in_tile = (i + 1 < planA.loads || !planA.last_guarded) ? true : (v < TM * KCH / 8);
            const int row = v / (KCH / 8), col = (v % (KCH / 8)) * 8;
            const bool ok = in_tile && (m0 + row < a.K);
            a_reg[i] = buffer_load_vec(rfilt, ok ? (uint32_t)((m0 + row) * a.Q + c0 * RS + col) * 2u : kOutOfRange);
        }
        const int slab = (img * a.C + c0) * a.HW;
        if constexpr (NAT) {
#pragma unroll
            for (int i = 0; i < LBN; ++i) {
                const int v = i * NT + tid;
                n_reg[i] = buffer_load_vec(rin, v < nvecN ? (uint32_t)slab * 2u + (uint32_t)v * 16u : kOutOfRange);
            }
        } else {
#pragma unroll
            for (int i = 0; i < LBT; ++i) {
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    b_reg[i][j] = buffer_load_elem<elem_t>(
                        rin, t_lds[i] >= 0 ? (uint32_t)(slab + t_goff[i] + j * a.HW) * 2u : kOutOfRange);
            }
        }
    };

    auto store_chunk = [&](int buf) {
        elem_t* As = As0 + buf * TM * LDA;
        elem_t* Bs = Bs0 + buf * b_elems;
#pragma unroll
        for (int i = 0; i < planA.loads; ++i) {
            const int v = i * NT + tid;
            const bool in_tile = (i + 1 < planA.loads || !planA.last_guarded) ? true : (v < TM * KCH / 8);
            const int row = v / (KCH / 8), col = (v % (KCH / 8)) * 8;
            if (in_tile) *(uint4*)&As[row * LDA + col] = a_reg[i];
        }
        if constexpr (NAT) {
#pragma unroll
            for (int i = 0; i < LBN; ++i) {
                const int v = i * NT + tid;
                if (v < nvecN) *(uint4*)&Nat[v * 8] = n_reg[i];
            }
        } else {
#pragma unroll
            for (int i = 0; i < LBT; ++i) {
                if (t_lds[i] >= 0) {
                    uint4 pk;
                    pk.x = (uint32_t)b_reg[i][0] | ((uint32_t)b_reg[i][1] << 16);
                    pk.y = (uint32_t)b_reg[i][2] | ((uint32_t)b_reg[i][3] << 16);
                    pk.z = (uint32_t)b_reg[i][4] | ((uint32_t)b_reg[i][5] << 16);
                    pk.w = (uint32_t)b_reg[i][6] | ((uint32_t)b_reg[i][7] << 16);
                    *(uint4*)&Bs[t_lds[i]] = pk;
                }
            }
        }
    };

    // LBN > 0: second half of the staging, raw LDS copy -> channel-innermost slab (after a barrier)
    auto transpose_chunk = [&](int buf) {
        elem_t* Bs = Bs0 + buf * b_elems;
#pragma unroll
        for (int i = 0; i < LBT; ++i) {
            if (t_lds[i] >= 0) {
                const elem_t* src = Nat + t_nat[i];
                uint4 pk;
                pk.x = (uint32_t)src[0 * a.HW] | ((uint32_t)src[1 * a.HW] << 16);
                pk.y = (uint32_t)src[2 * a.HW] | ((uint32_t)src[3 * a.HW] << 16);
                pk.z = (uint32_t)src[4 * a.HW] | ((uint32_t)src[5 * a.HW] << 16);
                pk.w = (uint32_t)src[6 * a.HW] | ((uint32_t)src[7 * a.HW] << 16);
                *(uint4*)&Bs[t_lds[i]] = pk;
            }
        }
    };

    // LDS position (times CP) of the window's first element for each pixel column of this lane
    int bpos[NBW];
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb) {
        const int n = (wn * NBW + nb) * 32 + li;
        uint32_t oyl, ox;
        a.dOW.divmod(n < npix ? (uint32_t)n : 0u, oyl, ox);
        bpos[nb] = ((int)oyl * PW + (int)ox) * CP;
    }
    const int chan0 = kw * 16 + g * 8;  // first of this lane's 8 channels inside the chunk

    typename mma_t::acc_t acc[TMB][NBW];
#pragma unroll
    for (int mb = 0; mb < TMB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mb][nb][v] = 0.0f;

    // A lane's filter operands of one chunk are 8 channels x R*S taps = 8*R*S consecutive 16-bit elements of its
    // filter row: they are fetched as R*S 16-byte LDS reads at the start of the chunk, and the operand of tap t
    // (element j*R*S + t for channel j) is then assembled in registers with one byte-permute per pair of channels.
    uint32_t araw[TMB][4 * RS];
    auto compute = [&](int buf, auto t0, auto t1) {
        constexpr int T0 = decltype(t0)::value, T1 = decltype(t1)::value;
        const elem_t* __restrict__ As = As0 + buf * TM * LDA + ((wm * TMB) * 32 + li) * LDA + chan0 * RS;
        const elem_t* __restrict__ Bs = Bs0 + buf * b_elems + chan0;
        if constexpr (T0 == 0) {
#pragma unroll
            for (int mb = 0; mb < TMB; ++mb)
#pragma unroll
                for (int i = 0; i < RS; ++i) {
                    const uint4 v = *(const uint4*)&As[mb * 32 * LDA + i * 8];
                    araw[mb][4 * i + 0] = v.x;
                    araw[mb][4 * i + 1] = v.y;
                    araw[mb][4 * i + 2] = v.z;
                    araw[mb][4 * i + 3] = v.w;
                }
        }
        // The patch operands of tap t + 1 are read before the products of tap t are issued (two register sets): a whole
        // tap's MFMAs cover the LDS latency.  Left to itself the compiler reads each operand just ahead of its use.
        uint4 bf[2][NBW];
        auto read_tap = [&](int t, int set) {
            const int toff = ((t / S) * PW + (t % S)) * CP;
#pragma unroll
            for (int nb = 0; nb < NBW; ++nb) bf[set][nb] = *(const uint4*)&Bs[bpos[nb] + toff];
        };
        read_tap(T0, 0);
#pragma unroll
        for (int t = T0; t < T1; ++t) {
            const int set = (t - T0) & 1;
            if (t + 1 < T1) read_tap(t + 1, set ^ 1);
            uint4 af[TMB];
#pragma unroll
            for (int mb = 0; mb < TMB; ++mb) {
                uint32_t d[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int pa = (2 * q) * RS + t, pb = (2 * q + 1) * RS + t;  // element positions of channels 2q, 2q+1
                    const uint32_t sel = (uint32_t)(2 * (pa & 1)) | ((uint32_t)(2 * (pa & 1) + 1) << 8) |
                                         ((uint32_t)(4 + 2 * (pb & 1)) << 16) | ((uint32_t)(5 + 2 * (pb & 1)) << 24);
                    d[q] = __builtin_amdgcn_perm(araw[mb][pb >> 1], araw[mb][pa >> 1], sel);
                }
                af[mb] = make_uint4(d[0], d[1], d[2], d[3]);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int mb = 0; mb < TMB; ++mb)
#pragma unroll
                for (int nb = 0; nb < NBW; ++nb) acc[mb][nb] = mma_t::run(af[mb], bf[set][nb], acc[mb][nb]);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    constexpr int TSPLIT = (RS * 5 + 8) / 9;
    typedef std::integral_constant<int, 0> tap_first;
    typedef std::integral_constant<int, TSPLIT> tap_mid;
    typedef std::integral_constant<int, RS> tap_last;

    if (chunk_begin < chunk_end) load_chunk(chunk_begin);  // in flight while the slabs are cleared
    // zero both patch slabs once: border and slack stay zero, real positions are overwritten by every chunk
    {
        uint4* z = (uint4*)Bs0;
        const int n16 = (2 * b_elems * (int)sizeof(elem_t)) / 16;
        for (int i = tid; i < n16; i += NT) z[i] = make_uint4(0, 0, 0, 0);
    }
    if (chunk_begin < chunk_end) {
        __syncthreads();  // zero fill done before the first real write
        store_chunk(0);
        if constexpr (NAT) {
            __syncthreads();
            transpose_chunk(0);
        }
        __syncthreads();
        int buf = 0;
        for (int chunk = chunk_begin; chunk < chunk_end; ++chunk) {
            const bool more = chunk + 1 < chunk_end;
            if (more) load_chunk(chunk + 1);
            compute(buf, tap_first{}, tap_mid{});
            if (more) store_chunk(buf ^ 1);  // the other buffer was last read before the previous barrier
            if constexpr (NAT) {
                if (more) {
                    __syncthreads();  // raw copy complete; it is not touched again before the barrier that ends this step
                    transpose_chunk(buf ^ 1);
                }
            }
            compute(buf, tap_mid{}, tap_last{});
            __syncthreads();
            buf ^= 1;
        }
    } else {
        __syncthreads();
    }

    // ---- add the KW channel-waves' partial sums in wave order, then bias + activation + rounding + store --------
    float* const red = (float*)smem_raw;  // [KW][32 rows][TNP]
    const bool split = a.nsplit > 1;
    const __amdgpu_buffer_rsrc_t rbias = make_rsrc(a.bias, a.bias ? (uint32_t)a.K * 4u : 0u);
    const __amdgpu_buffer_rsrc_t rout = make_rsrc(a.out, a.out_bytes);
    const __amdgpu_buffer_rsrc_t rws = make_rsrc(a.ws + (size_t)blockIdx.z * a.K * a.P, (uint32_t)a.K * a.P * 4u);
    const int pix0 = img * a.OHW + oy0 * a.OW;  // index of the band's first pixel in the [N*OH*OW] pixel axis
#pragma unroll
    for (int wmi = 0; wmi < WM; ++wmi) {
#pragma unroll
        for (int mb = 0; mb < TMB; ++mb) {
            if (wm == wmi) {
#pragma unroll
                for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        red[(kw * 32 + acc_row<32>(v, lane)) * TNP + (wn * NBW + nb) * 32 + li] = acc[mb][nb][v];
            }
            __syncthreads();
            if (a.pool) {
                // the band is the whole image: 3x3 stride-2 maxima of the summed block, then bias + activation + rounding
                // (all three are monotone, so this equals pooling the rounded activations)
                const int npool = a.POH * a.POW;
                for (int e = tid; e < 32 * npool; e += NT) {
                    uint32_t urow, upp, upy, upx;  // a.dX divides by POH*POW, a.dY by POW
                    a.dX.divmod((uint32_t)e, urow, upp);
                    a.dY.divmod(upp, upy, upx);
                    const int row = (int)urow, pp = (int)upp, py = (int)upy, px = (int)upx;
                    const int k = m0 + (wmi * TMB + mb) * 32 + row;
                    float m = -INFINITY;
#pragma unroll
                    for (int dy = 0; dy < 3; ++dy)
#pragma unroll
                        for (int dx = 0; dx < 3; ++dx) {
                            const int idx = row * TNP + (2 * py + dy) * a.OW + 2 * px + dx;
                            float x = red[idx];
#pragma unroll
                            for (int q = 1; q < KW; ++q) x += red[q * 32 * TNP + idx];
                            m = (x > m || (!a.relu && x != x)) ? x : m;  // NaN: dropped by the activation, else it is the result
                        }
                    const bool ok = k < a.K;
                    m += buffer_load_elem<float>(rbias, ok ? (uint32_t)k * 4u : kOutOfRange);
                    if (a.relu) m = m > 0.0f ? m : 0.0f;
                    buffer_store_elem<elem_t>(Prec<DT>::from_f32(m), rout, ok ? (uint32_t)((img * a.K + k) * npool + pp) * 2u : kOutOfRange);
                }
                __syncthreads();
                continue;
            }
            constexpr int NE = (32 * TNP + NT - 1) / NT;  // outputs of this 32-row block per thread
            float xs[NE], bs[NE];
#pragma unroll
            for (int j = 0; j < NE; ++j) {
                const int e = j * NT + tid;
                const int row = e / TNP;
                bs[j] = buffer_load_elem<float>(rbias, (e < 32 * TNP && !split) ? (uint32_t)(m0 + (wmi * TMB + mb) * 32 + row) * 4u
                                                                                : kOutOfRange);
            }
#pragma unroll
            for (int j = 0; j < NE; ++j) {
                const int e = j * NT + tid;
                const int idx = e < 32 * TNP ? e : 0;
                float x = red[idx];
#pragma unroll
                for (int q = 1; q < KW; ++q) x += red[q * 32 * TNP + idx];
                xs[j] = x;
            }
#pragma unroll
            for (int j = 0; j < NE; ++j) {
                const int e = j * NT + tid;
                const int row = e / TNP, col = e % TNP;
                const int k = m0 + (wmi * TMB + mb) * 32 + row;
                const bool ok = e < 32 * TNP && k < a.K && col < npix;
                if (split) {
                    buffer_store_elem<float>(xs[j], rws, ok ? (uint32_t)(k * a.P + pix0 + col) * 4u : kOutOfRange);
                } else {
                    float x = xs[j] + bs[j];
                    if (a.relu) x = x > 0.0f ? x : 0.0f;
                    buffer_store_elem<elem_t>(Prec<DT>::from_f32(x), rout,
                                              ok ? (uint32_t)((img * a.K + k) * a.OHW + oy0 * a.OW + col) * 2u : kOutOfRange);
                }
            }
            __syncthreads();
        }
    }
}

template <class CFG>
size_t wconv16_lds_bytes(int H, int W, int pad, int OH, int OW)
{
    const Wconv16Geom g = wconv16_geom<CFG>(W, pad, OH, OW);
    size_t pipe = 2 * sizeof(uint16_t) * ((size_t)CFG::TM * CFG::LDA + (size_t)g.npos * CFG::CP);
    if (CFG::LBN > 0) pipe += sizeof(uint16_t) * (((size_t)CFG::CB * H * W + 7) / 8 * 8);
    const size_t red = sizeof(float) * (size_t)CFG::RED_FLOATS;
    return pipe > red ? pipe : red;
}

template <class CFG>
hipError_t wconv16_launch(const Variant& v, ConvArgs& a, hipStream_t s)
{
    const size_t lds = wconv16_lds_bytes<CFG>(a.H, a.W, a.pad, a.OH, a.OW);
    const hipError_t e = ensure_dynamic_lds((const void*)wconv16_kernel<CFG>, lds);
    if (e != hipSuccess) return e;
    const Wconv16Geom g = wconv16_geom<CFG>(a.W, a.pad, a.OH, a.OW);
    const int total_chunks = a.C / CFG::CB;
    a.nsplit = v.split;
    a.steps_per_split = (total_chunks + v.split - 1) / v.split;
    dim3 grid((unsigned)(a.N * g.bands), (unsigned)((a.K + CFG::TM - 1) / CFG::TM), (unsigned)v.split);
    if (a.pool) {
        a.dX = make_fastdiv((uint32_t)(a.POH * a.POW));
        a.dY = make_fastdiv((uint32_t)a.POW);
    }
    hipLaunchKernelGGL(wconv16_kernel<CFG>, grid, dim3(CFG::NT), lds, s, a);
    return hipGetLastError();
}

template <class CFG>
bool wconv16_valid(const Variant& v, const conv_desc& d, int OH, int OW)
{
    if (d.dtype != CFG::DT || d.R != CFG::R || d.S != CFG::S || d.stride != 1) return false;
    if ((d.C % CFG::CB) != 0) return false;
    if (OW > CFG::TNP) return false;
    const Wconv16Geom g = wconv16_geom<CFG>(d.W, d.pad, OH, OW);
    if (CFG::LBN > 0) {
        if (g.bands != 1) return false;  // the raw copy is the whole image slab
        if ((long long)CFG::CB * d.H * d.W / 8 > (long long)CFG::NT * CFG::LBN) return false;
        if (((long long)d.C * d.H * d.W) % 8 != 0) return false;  // every image's slab must start 16-byte aligned
    }
    // every (input pixel of a band, channel octet) needs a staging slot
    const long long in_rows = g.in_rows < d.H ? g.in_rows : d.H;
    if (in_rows * d.W * (CFG::CB / 8) > (long long)CFG::NT * CFG::LBT) return false;
    if (wconv16_lds_bytes<CFG>(d.H, d.W, d.pad, OH, OW) > 160 * 1024) return false;
    // at least 60 % of the pixel columns computed over the image must be real
    if ((long long)OH * OW * 10 < (long long)g.bands * CFG::TNP * 6) return false;
    const int chunks = d.C / CFG::CB;
    if (v.split > 1 && chunks < 2 * v.split) return false;
    const long long P = (long long)d.N * OH * OW;
    if (v.split > 1 && (long long)d.K * P * 4 >= (1LL << 32)) return false;
    if (CFG::TM > 32 && d.K < CFG::TM) return false;
    if (d.K > 65535LL * CFG::TM || (long long)d.N * g.bands > 2147483647LL) return false;
    // the fused max-pool reads its windows from the workgroup's own tile: one band per image, no partial sums elsewhere
    if ((d.flags & CONV_FLAG_MAXPOOL_3X3S2) && (g.bands != 1 || v.split > 1)) return false;
    return true;
}

template <class CFG>
void wconv16_register(std::vector<Variant>& out, std::initializer_list<int> splits)
{
    for (int sk : splits) {
        Variant v;
        char buf[160];
        snprintf(buf, sizeof buf, "wconv_%s_%dx%d_M%dN%dC%d_w%dx%dx%d%s", dtype_name(CFG::DT), CFG::R, CFG::S, CFG::TM,
                 CFG::TNP, CFG::CB, CFG::KW, CFG::WM, CFG::WN, CFG::LBN > 0 ? "_img" : "");
        v.name = buf;
        if (sk > 1) v.name += "_sk" + std::to_string(sk);
        v.dtype = CFG::DT;
        v.split = sk;
        v.tm = CFG::TM;
        v.tn = CFG::TNP;
        v.tk = CFG::KCH;
        v.threads = CFG::NT;
        v.family = FAM_WINDOW;
        v.specificity = 4;
        v.traits = (CFG::LBN > 0 ? TRAIT_WHOLE_IMAGE : 0u) | TRAIT_POOL_EPILOGUE;
        v.valid = &wconv16_valid<CFG>;
        v.launch = &wconv16_launch<CFG>;
        out.push_back(v);
    }
}

}  // namespace convfwd
