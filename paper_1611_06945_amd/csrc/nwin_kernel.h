// Window-reuse convolution for stride-1 layers on channel-innermost tensors, fp16 / bf16 storage.
//
// The 16-bit window kernel has to transpose its NCHW input into [position][channel] order on the way into LDS,
// because a lane feeds 8 consecutive channels to each 32x32x16 MFMA.  When the graph keeps activations channel-innermost
// (the paper's explicit data-format conversions, Section 3 "Graph-level Optimizations") that order is what global memory
// already holds:
//     in   [N][H][W][C]      filt [K][R][S][C]      out [N][OH][OW][K] or [N][K][OH][OW]
// so the slab of one chunk of CB channels is copied with plain 16-byte loads and stores -- every position's CB channels
// are 2*CB contiguous bytes -- and the filter slab [TM][R*S][CB] likewise; a lane's operands for tap (r,s) are one
// 16-byte LDS read each (filter: row, tap, its 8 channels; patch: window origin + r*PW + s, its 8 channels).
// Everything else is the organisation of the NCHW window kernel: a workgroup owns TM output channels x a band of output
// rows of one image, KW waves split the chunk's channels, WN waves split the pixel blocks, partial sums of the KW
// channel-waves are added in wave order through LDS, then bias + activation + rounding + store in either output format.
#pragma once

#include <type_traits>

#include "wconv16_kernel.h"

namespace convfwd {

template <int DT_, int R_, int S_, int KW_, int WM_, int TMB_, int WN_, int NBW_, int LBT_>
struct NwinCfg {
    static_assert(DT_ == CONV_F16 || DT_ == CONV_BF16, "16-bit storage only");
    static constexpr int DT = DT_, R = R_, S = S_, KW = KW_, WM = WM_, TMB = TMB_, WN = WN_, NBW = NBW_, LBT = LBT_;
    static constexpr int RS = R * S;
    static constexpr int NT = 64 * KW * WM * WN;
    static constexpr int CB = 16 * KW;                 // channels per chunk
    static constexpr int CV = CB / 8;                  // 16-byte vectors per position / per (row, tap)
    static constexpr int TM = 32 * TMB * WM;           // output channels per workgroup
    static constexpr int TNP = 32 * NBW * WN;          // pixel columns per workgroup
    static constexpr int LDA = RS * CB + 8;            // filter slab row pitch (16-bit elements)
    static constexpr int CP = CB + 8;                  // channel pitch of one LDS position
    static constexpr int A_VECS = TM * RS * CV;
    static constexpr CoopPlan planA = coop_plan(NT, A_VECS);
    static constexpr int RP = TNP + 1;                 // row pitch of the reduction buffer: odd, so that reads along either axis spread over the banks
    static constexpr int RED_FLOATS = KW * 32 * RP;    // one 32-row block at a time
};

template <class CFG>
__global__ __launch_bounds__(CFG::NT) void nwin_kernel(ConvArgs a)
{
    typedef uint16_t elem_t;
    constexpr int DT = CFG::DT, R = CFG::R, S = CFG::S, RS = CFG::RS, KW = CFG::KW, WM = CFG::WM, TMB = CFG::TMB;
    constexpr int WN = CFG::WN, NBW = CFG::NBW, LBT = CFG::LBT, NT = CFG::NT, CB = CFG::CB, CV = CFG::CV, TM = CFG::TM;
    constexpr int TNP = CFG::TNP, LDA = CFG::LDA, CP = CFG::CP, A_VECS = CFG::A_VECS, RP = CFG::RP;
    constexpr CoopPlan planA = CFG::planA;
    typedef Mma<DT, 32> mma_t;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];

    const Wconv16Geom geo = wconv16_geom<CFG>(a.W, a.pad, a.OH, a.OW);
    const int PW = a.W + 2 * a.pad;
    elem_t* const As0 = (elem_t*)smem_raw;              // [2][TM*LDA]
    elem_t* const Bs0 = As0 + 2 * TM * LDA;             // [2][npos*CP]
    const int b_elems = geo.npos * CP;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kw = wave % KW, wn = (wave / KW) % WN, wm = wave / (KW * WN);
    const int li = lane & 31, g = lane >> 5;
    const int chan0 = kw * 16 + g * 8;  // first of this lane's 8 channels inside the chunk

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

    // ---- staging plans (the same for every chunk: only the channel offset moves) -------------------------------------
    // patch slab: task = (input position of the band, 16-byte vector of the chunk's channels)
    const int iy_first = oy0 - a.pad;
    const int iy_lo = iy_first < 0 ? 0 : iy_first;
    int iy_hi = iy_first + bh + R - 1;
    if (iy_hi > a.H) iy_hi = a.H;
    const int ntask = (iy_hi - iy_lo) * a.W * CV;
    uint32_t t_goff[LBT];  // byte offset of the vector for chunk 0, or out of range
    int t_lds[LBT];        // element index in the LDS slab, or -1
#pragma unroll
    for (int i = 0; i < LBT; ++i) {
        const int t = i * NT + tid;
        const bool ok = t < ntask;
        const int pos = ok ? t / CV : 0, v8 = t % CV;
        uint32_t y, x;
        a.dW.divmod((uint32_t)pos, y, x);
        t_goff[i] = ok ? (uint32_t)((((img * a.H + iy_lo + (int)y) * a.W + (int)x) * a.C + v8 * 8)) * 2u : kOutOfRange;
        t_lds[i] = ok ? ((iy_lo - iy_first + (int)y) * PW + (int)x + a.pad) * CP + v8 * 8 : -1;
    }
    // filter slab: vector = (row, tap, 16-byte vector of the chunk's channels)
    uint32_t f_goff[planA.loads];
    int f_lds[planA.loads];
#pragma unroll
    for (int i = 0; i < planA.loads; ++i) {
        const int v = i * NT + tid;
        const bool in_tile = (i + 1 < planA.loads || !planA.last_guarded) ? true : (v < A_VECS);
        const int row = v / (RS * CV), rem = v % (RS * CV), tap = rem / CV, v8 = rem % CV;
        const bool ok = in_tile && (m0 + row < a.K);
        f_goff[i] = ok ? (uint32_t)(((m0 + row) * RS + tap) * a.C + v8 * 8) * 2u : kOutOfRange;
        f_lds[i] = in_tile ? row * LDA + tap * CB + v8 * 8 : -1;
    }

    uint4 a_reg[planA.loads], b_reg[LBT];
    auto load_chunk = [&](int chunk) {
        const uint32_t c_bytes = (uint32_t)(chunk * CB) * 2u;
#pragma unroll
        for (int i = 0; i < planA.loads; ++i) a_reg[i] = buffer_load_vec(rfilt, f_goff[i] == kOutOfRange ? kOutOfRange : f_goff[i] + c_bytes);
#pragma unroll
        for (int i = 0; i < LBT; ++i) b_reg[i] = buffer_load_vec(rin, t_goff[i] == kOutOfRange ? kOutOfRange : t_goff[i] + c_bytes);
    };
    auto store_chunk = [&](int buf) {
        elem_t* As = As0 + buf * TM * LDA;
        elem_t* Bs = Bs0 + buf * b_elems;
#pragma unroll
        for (int i = 0; i < planA.loads; ++i)
            if (f_lds[i] >= 0) *(uint4*)&As[f_lds[i]] = a_reg[i];
#pragma unroll
        for (int i = 0; i < LBT; ++i)
            if (t_lds[i] >= 0) *(uint4*)&Bs[t_lds[i]] = b_reg[i];
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

    typename mma_t::acc_t acc[TMB][NBW];
#pragma unroll
    for (int mb = 0; mb < TMB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mb][nb][v] = 0.0f;

    auto compute = [&](int buf, auto t0, auto t1) {
        constexpr int T0 = decltype(t0)::value, T1 = decltype(t1)::value;
        const elem_t* __restrict__ As = As0 + buf * TM * LDA + ((wm * TMB) * 32 + li) * LDA + chan0;
        const elem_t* __restrict__ Bs = Bs0 + buf * b_elems + chan0;
        // The operands of tap t + 1 are read before the products of tap t are issued (two register sets): a whole tap's
        // MFMAs cover the LDS latency.  Left to itself the compiler reads each operand just ahead of its use.
        uint4 af[2][TMB], bf[2][NBW];
        auto read_tap = [&](int t, int set) {
            const int r = t / S, s = t % S;
#pragma unroll
            for (int mb = 0; mb < TMB; ++mb) af[set][mb] = *(const uint4*)&As[mb * 32 * LDA + t * CB];
            const int toff = (r * PW + s) * CP;
#pragma unroll
            for (int nb = 0; nb < NBW; ++nb) bf[set][nb] = *(const uint4*)&Bs[bpos[nb] + toff];
        };
        read_tap(T0, 0);
#pragma unroll
        for (int t = T0; t < T1; ++t) {
            const int set = (t - T0) & 1;
            if (t + 1 < T1) read_tap(t + 1, set ^ 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int mb = 0; mb < TMB; ++mb)
#pragma unroll
                for (int nb = 0; nb < NBW; ++nb) acc[mb][nb] = mma_t::run(af[set][mb], bf[set][nb], acc[mb][nb]);
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
        // The registers are free again: the next chunk's loads start now and have a whole chunk's products to arrive,
        // not the part of one that precedes their store.  Loads are unconditional (past the last chunk they fetch the
        // neighbouring channels or fall outside the tensors; the data is not used): a conditional load makes every
        // later wait assume the worst.
        load_chunk(chunk_begin + 1);
        __syncthreads();
        int buf = 0;
        for (int chunk = chunk_begin; chunk < chunk_end; ++chunk) {
            const bool more = chunk + 1 < chunk_end;
            compute(buf, tap_first{}, tap_mid{});
            if (more) store_chunk(buf ^ 1);  // the other buffer was last read before the previous barrier
            load_chunk(chunk + 2);
            compute(buf, tap_mid{}, tap_last{});
            __syncthreads();
            buf ^= 1;
        }
    } else {
        __syncthreads();
    }

    // ---- add the KW channel-waves' partial sums in wave order, then bias + activation + rounding + store --------
    float* const red = (float*)smem_raw;  // [KW][32 rows][RP]
    const bool split = a.nsplit > 1;
    const bool onhwc = a.out_nhwc != 0 && !split;
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
                        red[(kw * 32 + acc_row<32>(v, lane)) * RP + (wn * NBW + nb) * 32 + li] = acc[mb][nb][v];
            }
            __syncthreads();
            if (a.pool) {
                // the band is the whole image: 3x3 stride-2 maxima of the summed block, then bias + activation + rounding
                // (all three are monotone, so this equals pooling the rounded activations)
                const int npool = a.POH * a.POW;
                for (int e = tid; e < 32 * npool; e += NT) {
                    uint32_t qrow, qpp, upy, upx;  // a.dX divides by POH*POW, a.dY by POW
                    a.dX.divmod((uint32_t)e, qrow, qpp);
                    const int row = onhwc ? (e & 31) : (int)qrow, pp = onhwc ? (e >> 5) : (int)qpp;
                    a.dY.divmod((uint32_t)pp, upy, upx);
                    const int py = (int)upy, px = (int)upx;
                    const int k = m0 + (wmi * TMB + mb) * 32 + row;
                    float m = -INFINITY;
#pragma unroll
                    for (int dy = 0; dy < 3; ++dy)
#pragma unroll
                        for (int dx = 0; dx < 3; ++dx) {
                            const int idx = row * RP + (2 * py + dy) * a.OW + 2 * px + dx;
                            float x = red[idx];
#pragma unroll
                            for (int q = 1; q < KW; ++q) x += red[q * 32 * RP + idx];
                            m = (x > m || (!a.relu && x != x)) ? x : m;  // NaN: dropped by the activation, else it is the result
                        }
                    const bool ok = k < a.K;
                    m += buffer_load_elem<float>(rbias, ok ? (uint32_t)k * 4u : kOutOfRange);
                    if (a.relu) m = m > 0.0f ? m : 0.0f;
                    const uint32_t o = onhwc ? (uint32_t)((img * npool + pp) * a.K + k) : (uint32_t)((img * a.K + k) * npool + pp);
                    buffer_store_elem<elem_t>(Prec<DT>::from_f32(m), rout, ok ? o * 2u : kOutOfRange);
                }
                __syncthreads();
                continue;
            }
            constexpr int NE = (32 * TNP + NT - 1) / NT;  // outputs of this 32-row block per thread
#pragma unroll
            for (int j = 0; j < NE; ++j) {
                const int e = j * NT + tid;
                // channel-planar output: consecutive threads take consecutive pixels; channel-innermost: consecutive channels
                const int row = onhwc ? (e & 31) : e / TNP, col = onhwc ? (e >> 5) : e % TNP;
                const int k = m0 + (wmi * TMB + mb) * 32 + row;
                const bool ok = e < 32 * TNP && k < a.K && col < npix;
                const int idx = ok ? row * RP + col : 0;
                float x = red[idx];
#pragma unroll
                for (int q = 1; q < KW; ++q) x += red[q * 32 * RP + idx];
                if (split) {
                    buffer_store_elem<float>(x, rws, ok ? (uint32_t)(k * a.P + pix0 + col) * 4u : kOutOfRange);
                } else {
                    x += buffer_load_elem<float>(rbias, ok ? (uint32_t)k * 4u : kOutOfRange);
                    if (a.relu) x = x > 0.0f ? x : 0.0f;
                    const uint32_t o = onhwc ? (uint32_t)((pix0 + col) * a.K + k) : (uint32_t)((img * a.K + k) * a.OHW + oy0 * a.OW + col);
                    buffer_store_elem<elem_t>(Prec<DT>::from_f32(x), rout, ok ? o * 2u : kOutOfRange);
                }
            }
            __syncthreads();
        }
    }
}

template <class CFG>
size_t nwin_lds_bytes(int W, int pad, int OH, int OW)
{
    const Wconv16Geom g = wconv16_geom<CFG>(W, pad, OH, OW);
    const size_t pipe = 2 * sizeof(uint16_t) * ((size_t)CFG::TM * CFG::LDA + (size_t)g.npos * CFG::CP);
    const size_t red = sizeof(float) * (size_t)CFG::RED_FLOATS;
    return pipe > red ? pipe : red;
}

template <class CFG>
hipError_t nwin_launch(const Variant& v, ConvArgs& a, hipStream_t s)
{
    const size_t lds = nwin_lds_bytes<CFG>(a.W, a.pad, a.OH, a.OW);
    const hipError_t e = ensure_dynamic_lds((const void*)nwin_kernel<CFG>, lds);
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
    hipLaunchKernelGGL(nwin_kernel<CFG>, grid, dim3(CFG::NT), lds, s, a);
    return hipGetLastError();
}

template <class CFG>
bool nwin_valid(const Variant& v, const conv_desc& d, int OH, int OW)
{
    if (d.dtype != CFG::DT || d.R != CFG::R || d.S != CFG::S || d.stride != 1) return false;
    if (!(d.flags & CONV_FLAG_IN_NHWC) || !(d.flags & CONV_FLAG_FILT_KRSC)) return false;
    if ((d.C % CFG::CB) != 0) return false;
    if (OW > CFG::TNP) return false;
    const Wconv16Geom g = wconv16_geom<CFG>(d.W, d.pad, OH, OW);
    // every (input position of a band, 16-byte vector) needs a staging slot
    const long long in_rows = g.in_rows < d.H ? g.in_rows : d.H;
    if (in_rows * d.W * CFG::CV > (long long)CFG::NT * CFG::LBT) return false;
    if (nwin_lds_bytes<CFG>(d.W, d.pad, OH, OW) > 160 * 1024) return false;
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
void nwin_register(std::vector<Variant>& out, std::initializer_list<int> splits)
{
    for (int sk : splits) {
        Variant v;
        char buf[160];
        snprintf(buf, sizeof buf, "nhwc_win_%s_%dx%d_M%dN%dC%d_w%dx%dx%d", dtype_name(CFG::DT), CFG::R, CFG::S, CFG::TM, CFG::TNP,
                 CFG::CB, CFG::KW, CFG::WM, CFG::WN);
        v.name = buf;
        if (sk > 1) v.name += "_sk" + std::to_string(sk);
        v.dtype = CFG::DT;
        v.split = sk;
        v.tm = CFG::TM;
        v.tn = CFG::TNP;
        v.tk = CFG::CB * CFG::RS;
        v.threads = CFG::NT;
        v.family = FAM_NHWC;
        v.specificity = 5;
        v.traits = TRAIT_WINDOW_TILES | TRAIT_POOL_EPILOGUE;
        v.valid = &nwin_valid<CFG>;
        v.launch = &nwin_launch<CFG>;
        out.push_back(v);
    }
}

}  // namespace convfwd
