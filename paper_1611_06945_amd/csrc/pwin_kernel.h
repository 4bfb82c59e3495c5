// Window-reuse convolution for stride-1 layers, fp16 / bf16 storage, with the filters handed over in MFMA operand
// order ("packed": an explicit data-format conversion done once, ahead of time, in the sense of the paper's Section 3
// "Graph-level Optimizations" -- at inference the weights are constants).
//
// What bounds a 16-bit MFMA kernel on this device is operand delivery, not arithmetic: a CU issues one 32x32x16 MFMA
// every 8 cycles and each one consumes 1 KB of filter and 1 KB of patch operand, while LDS delivers 128 B and the
// vector memory path 64 B per cycle.  So
//   * the two operands come over the two different paths.  A filter fragment is used by exactly one wave, once per
//     chunk: staging it in LDS would only add a write and a read.  Packed filters are stored as the 1 KB fragments
//     the MFMA consumes ([32-row block][16-channel group][tap][lane][8 channels]), so a fragment is ONE coalesced
//     16-byte-per-lane load from L2 straight into the registers of the wave that multiplies with it, issued AD taps
//     ahead through a ring of AD register slots;
//   * the patch operand is read from an LDS copy of the input (every tap of the window is the same slab at a constant
//     offset: overlapping windows share the copy; paper, Section 5), and each fragment read feeds TMB = 2 MFMAs (two
//     32-row blocks per wave), which halves the LDS traffic per MFMA;
//   * KW waves split the chunk's channels (16 each) so that even a 64 x 96 output tile keeps four SIMDs busy; their
//     partial sums are added in wave order through LDS at the end (deterministic), then bias + activation + one
//     rounding + store.
// The pixel axis is linear over (image, row, column): a tile is any run of TNP pixels and may straddle images.  The
// slab addresses input elements by a position in a stack of all images that SHARES the zero border between
// neighbours -- row pitch W + pad, image pitch H + pad rows -- so the operand of pixel p at tap (r,s) sits at
// base(p) + r*(W+pad) + s whatever image p belongs to; a position in a shared border is written as zero.
// Workgroups are dealt to the 8 XCDs round-robin by the hardware; the ids one XCD receives are mapped to a contiguous
// run of pixel tiles of (mostly) one channel tile, so the workgroups of an XCD stream the same filter fragments
// through its L2 at about the same time.
#pragma once

#include <type_traits>
#include <utility>

#include "igemm_kernel.h"

#ifndef PWIN_EXP
#define PWIN_EXP 0
#endif

namespace convfwd {

template <int DT_, int R_, int S_, int KW_, int WN_, int TMB_, int NBW_, int AD_, int LBT_, bool ALIGN8_ = false>
struct PwinCfg {
    static_assert(DT_ == CONV_F16 || DT_ == CONV_BF16, "16-bit storage only");
    static constexpr int DT = DT_, R = R_, S = S_, KW = KW_, WN = WN_, TMB = TMB_, NBW = NBW_, AD = AD_, LBT = LBT_;
    // ALIGN8: widen the slab's row pitch until it equals the output row length modulo 8.  Eight lanes' 16-byte reads are
    // served per cycle and fall on distinct banks when their positions differ modulo 8; consecutive pixels are
    // consecutive positions except across a row end, where the pitch minus the row length is skipped -- a multiple of 8
    // keeps every read conflict free, at the price of more (zero) positions to stage.
    static constexpr bool ALIGN8 = ALIGN8_;
    static constexpr int RS = R * S;
    static_assert(RS % AD == 0, "the filter-fragment ring must divide the taps of a chunk");
    static constexpr int NT = 64 * KW * WN;
    static constexpr int CB = 16 * KW;        // channels per chunk
    static constexpr int CV = CB / 8;         // 16-byte vectors per slab position
    static_assert((CV & (CV - 1)) == 0, "KW must be a power of two");
    static constexpr int TM = 32 * TMB;       // output channels per workgroup
    static constexpr int TNP = 32 * NBW * WN; // pixels per workgroup
    static constexpr int CP = CB + 8;         // channel pitch of one slab position (16-bit elements)
    static constexpr int SLOTS = LBT * NT / CV;  // slab positions one buffer holds: every thread stages LBT vectors
    static constexpr int SLAB_ELEMS = SLOTS * CP;
    // Reduction buffer [KW][pixel][RBP]: the rows (channels) of one pixel are contiguous, so an accumulator's four
    // consecutive rows go out as one 16-byte LDS write and come back as 16-byte reads; RBP = RB + 4 floats makes the
    // pixel pitch = 4 banks (mod 64): 16 lanes cover all banks.  RB = rows summed per pass: all when that fits, else 32.
    static constexpr int RB = ((size_t)KW * TNP * (TM + 4) * 4 <= 160 * 1024) ? TM : 32;
    static constexpr int RBP = RB + 4;
    static constexpr size_t LDS_PIPE = 2 * sizeof(uint16_t) * (size_t)SLAB_ELEMS;
    static constexpr size_t LDS_RED = sizeof(float) * ((size_t)KW * TNP * RBP + RB);  // partial tiles + the bias values of the pass
    static constexpr size_t LDS_BYTES = LDS_PIPE > LDS_RED ? LDS_PIPE : LDS_RED;
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
};

// f(integral_constant<int, 0>{}), ..., f(integral_constant<int, N-1>{}): a loop whose index is a constant inside the
// body (register arrays indexed by it stay in registers, per-iteration decisions are `if constexpr`).
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

struct PwinGeom {
    int PWs, PHs;  // row pitch and image pitch (in rows) of the stacked position space
    int PT, MT;    // pixel tiles, channel tiles
    int span;      // most slab positions any pixel tile needs
};

template <class CFG>
inline PwinGeom pwin_geom(int N, int H, int W, int K, int pad, int OH, int OW)
{
    PwinGeom g;
    g.PWs = W + pad;
    if (CFG::ALIGN8) g.PWs += (((OW - g.PWs) % 8) + 8) % 8;
    g.PHs = H + pad;
    const long long P = (long long)N * OH * OW;
    g.PT = (int)((P + CFG::TNP - 1) / CFG::TNP);
    g.MT = (K + CFG::TM - 1) / CFG::TM;
    // a tile's first and last pixel are at most this many output rows / images apart
    long long rows = (CFG::TNP - 1 + OW - 1) / OW;
    if (rows > (long long)N * OH - 1) rows = (long long)N * OH - 1;
    long long imgs = (rows + OH - 1) / OH;
    if (imgs > N - 1) imgs = N - 1;
    const long long span = (rows + imgs * (g.PHs - OH)) * g.PWs + (OW - 1) + (long long)(CFG::R - 1) * g.PWs + CFG::S;
    g.span = span > 0x7fffffff ? 0x7fffffff : (int)span;
    return g;
}

// a.dX divides by PT, a.dY by W + pad, a.dZ by H + pad (set by the launcher)
template <class CFG>
__global__ __launch_bounds__(CFG::NT) void pwin_kernel(ConvArgs a)
{
    typedef uint16_t elem_t;
    constexpr int DT = CFG::DT, R = CFG::R, S = CFG::S, RS = CFG::RS, KW = CFG::KW, WN = CFG::WN, TMB = CFG::TMB;
    constexpr int NBW = CFG::NBW, AD = CFG::AD, LBT = CFG::LBT, NT = CFG::NT, CB = CFG::CB, CV = CFG::CV, TM = CFG::TM;
    constexpr int TNP = CFG::TNP, CP = CFG::CP, SLAB_ELEMS = CFG::SLAB_ELEMS, RBP = CFG::RBP, RB = CFG::RB;
    typedef Mma<DT, 32> mma_t;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    elem_t* const Bs0 = (elem_t*)smem_raw;  // [2][SLOTS][CP]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kw = wave % KW, wn = wave / KW;
    const int li = lane & 31, g = lane >> 5;
#if PWIN_EXP & 16
    unsigned long long* const tstamp = (unsigned long long*)a.ws + (size_t)blockIdx.x * 8;
    if (tid == 0 && a.ws) tstamp[0] = wall_clock64();
#endif

    // ---- which tile: ids b, b+8, b+16, ... run on one XCD; give each XCD a contiguous run of logical tiles ---------
    const int PT = (int)a.dX.d, PWs = (int)a.dY.d, PHs = (int)a.dZ.d;
    const int MT = (a.K + TM - 1) / TM;
    const int T = MT * PT;
    int logical;
    {
        const int b = blockIdx.x, x = b & 7, q = b >> 3;
        const int per = T >> 3, rem = T & 7;
        logical = x * per + (x < rem ? x : rem) + q;
    }
    uint32_t mt_u, pt_u;
    a.dX.divmod((uint32_t)logical, mt_u, pt_u);
    const int m0 = (int)mt_u * TM;
    const int p0 = (int)pt_u * TNP;
    const int plast = (p0 + TNP < a.P ? p0 + TNP : a.P) - 1;

    auto base_pos = [&](int p) {
        uint32_t n, pix, oy, ox;
        a.dOHW.divmod((uint32_t)p, n, pix);
        a.dOW.divmod(pix, oy, ox);
        return ((int)n * PHs + (int)oy) * PWs + (int)ox;
    };
    const int lo = base_pos(p0);
    const int nposw = base_pos(plast) + (R - 1) * PWs + S - lo;  // slab positions this tile needs

    const __amdgpu_buffer_rsrc_t rin = make_rsrc(a.in, a.in_bytes);
    const __amdgpu_buffer_rsrc_t rfilt = make_rsrc(a.filt, a.filt_bytes);

    // ---- filter fragments: ring of AD taps, each TMB fragments of 1 KB loaded straight from the packed tensor ------
    // (the first AD taps are requested before anything else: their latency covers the index arithmetic below)
    const int C16 = a.C >> 4;
    const uint32_t a_lane = (uint32_t)lane * 16u;
    const uint32_t a_mb_stride = (uint32_t)C16 * RS * 1024u;
    uint32_t a_soff = (uint32_t)((mt_u * TMB) * C16 + kw) * (RS * 1024u);  // chunk 0, tap 0, block 0 of this wave
    uint4 ar[AD][TMB];
    auto load_a = [&](auto slot_c, uint32_t soff) {
        constexpr int slot = decltype(slot_c)::value;
#pragma unroll
        for (int mb = 0; mb < TMB; ++mb) {
            const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rfilt, (int)a_lane, (int)(soff + (uint32_t)mb * a_mb_stride), 0);
            ar[slot][mb] = make_uint4(v.x, v.y, v.z, v.w);
        }
    };
    static_for<AD>([&](auto ic) { load_a(ic, a_soff + (uint32_t)decltype(ic)::value * 1024u); });

    // ---- staging plan of the slab (the same for every chunk: only the channel offset moves) ------------------------
    // task t = (slab position t / CV, 16-byte vector t % CV of the chunk's channels)
    uint32_t t_goff[LBT];
#pragma unroll
    for (int i = 0; i < LBT; ++i) {
        const int t = i * NT + tid;
        const int j = t / CV, v8 = t % CV;
        uint32_t Y, X, n, yy;
        a.dY.divmod((uint32_t)(lo + j), Y, X);
        a.dZ.divmod(Y, n, yy);
        const bool ok = j < nposw && (int)X >= a.pad && (int)X < a.pad + a.W && (int)yy >= a.pad && (int)n < a.N;
        t_goff[i] = ok ? (uint32_t)((((int)n * a.H + (int)yy - a.pad) * a.W + (int)X - a.pad) * a.C + v8 * 8) * 2u : kOutOfRange;
    }
    uint4 b_reg[LBT];
    auto load_slab = [&](int chunk) {
        const uint32_t c_bytes = (uint32_t)(chunk * CB) * 2u;
#pragma unroll
        for (int i = 0; i < LBT; ++i) b_reg[i] = buffer_load_vec(rin, t_goff[i] == kOutOfRange ? kOutOfRange : t_goff[i] + c_bytes);
    };
    auto store_slab = [&](int buf) {
        elem_t* Bs = Bs0 + buf * SLAB_ELEMS;
#pragma unroll
        for (int i = 0; i < LBT; ++i) {
            const int t = i * NT + tid;
            *(uint4*)&Bs[(t / CV) * CP + (t % CV) * 8] = b_reg[i];
        }
    };

    // slab element index of the window origin of each of this lane's pixel columns, at this lane's 8 channels
    int bpos[NBW];
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb) {
        const int p = p0 + (wn * NBW + nb) * 32 + li;
        bpos[nb] = (base_pos(p < a.P ? p : plast) - lo) * CP + kw * 16 + g * 8;
    }
    const int rowoff = PWs * CP;

    typename mma_t::acc_t acc[TMB][NBW];
#pragma unroll
    for (int mb = 0; mb < TMB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mb][nb][v] = 0.0f;

    const int nchunks = a.C / CB;

    // ---- prologue ---------------------------------------------------------------------------------------------------
    load_slab(0);
    store_slab(0);
    load_slab(1);  // unconditional: with a single chunk the data is never used
    __syncthreads();

#if PWIN_EXP & 16
    if (tid == 0 && a.ws) tstamp[1] = wall_clock64();
#endif
    uint4 bf[2][NBW];
    auto read_tap = [&](const elem_t* Bs, int r, int s, int set) {
        const int toff = r * rowoff + s * CP;
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb) bf[set][nb] = *(const uint4*)&Bs[bpos[nb] + toff];
    };
    read_tap(Bs0, 0, 0, 0);

    constexpr int TSTORE = RS / 2;  // tap after which the next chunk's slab goes to LDS
    constexpr uint32_t kChunkStep = (uint32_t)KW * RS * 1024u;
    int buf = 0;
    // One chunk.  STORE: another chunk follows (its slab is written to the other buffer at tap TSTORE, and the barrier
    // before the last tap publishes it); LOAD: a chunk follows that one (its slab is requested); the last chunk does
    // neither and requests no filter fragments past its own taps.  The three forms are separate straight-line code: a
    // load under a condition would make every later wait assume it was skipped and wait for too much.
    auto do_chunk = [&](auto store_c, auto load_c, int chunk) {
        constexpr bool STORE = decltype(store_c)::value, LOAD = decltype(load_c)::value;
        const elem_t* Bs = Bs0 + buf * SLAB_ELEMS;
        const elem_t* Bn = Bs0 + (buf ^ 1) * SLAB_ELEMS;
        static_for<RS>([&](auto tc) {
            constexpr int t = decltype(tc)::value, cur = t & 1, slot = t % AD;
            if constexpr (t + 1 < RS) {
                if constexpr (!(PWIN_EXP & 4)) read_tap(Bs, (t + 1) / S, (t + 1) % S, cur ^ 1);
            } else if constexpr (STORE) {
                // every wave holds its operands of the chunk's last tap in registers: the other buffer (stored at tap
                // TSTORE by everyone) becomes readable, and this one may be overwritten from the next chunk's tap
                // TSTORE on
                if constexpr (!(PWIN_EXP & 8)) __syncthreads();
                if constexpr (!(PWIN_EXP & 4)) read_tap(Bn, 0, 0, cur ^ 1);
            } else {
                // last tap of the last chunk: once every wave holds its last operands the slabs are dead, and the
                // reduction buffer that overlays them may be written
                __syncthreads();
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int mb = 0; mb < TMB; ++mb)
#pragma unroll
                for (int nb = 0; nb < NBW; ++nb) acc[mb][nb] = mma_t::run(ar[slot][mb], bf[cur][nb], acc[mb][nb]);
            // the slot is free once its MFMAs are issued: fetch the fragments of the tap AD ahead
            constexpr int ta = t + AD;
            if constexpr (!(PWIN_EXP & 1) && (ta < RS || STORE))
                load_a(std::integral_constant<int, slot>{},
                       a_soff + (ta < RS ? (uint32_t)ta * 1024u : kChunkStep + (uint32_t)(ta - RS) * 1024u));
            if constexpr (t == TSTORE && !(PWIN_EXP & 2)) {
                if constexpr (STORE) store_slab(buf ^ 1);
                if constexpr (LOAD) load_slab(chunk + 2);
            }
            __builtin_amdgcn_sched_barrier(0);
        });
        if constexpr ((RS & 1) != 0) {
#pragma unroll
            for (int nb = 0; nb < NBW; ++nb) bf[0][nb] = bf[1][nb];
        }
        buf ^= 1;
        a_soff += kChunkStep;
    };
    {
        int chunk = 0;
        for (; chunk + 2 < nchunks; ++chunk) do_chunk(std::true_type{}, std::true_type{}, chunk);
        if (chunk + 1 < nchunks) do_chunk(std::true_type{}, std::false_type{}, chunk++);
        do_chunk(std::false_type{}, std::false_type{}, chunk);
    }

    // ---- add the KW channel-waves' partial sums in wave order, then bias + activation + rounding + store -----------
    // (after the barrier in the last chunk's last tap no wave reads the slabs any more: the buffer is reused at once)
#if PWIN_EXP & 16
    if (tid == 0 && a.ws) tstamp[2] = wall_clock64();
#endif
    float* const red = (float*)smem_raw;  // [KW][TNP][RBP]
    const bool onhwc = a.out_nhwc != 0;
    const __amdgpu_buffer_rsrc_t rbias = make_rsrc(a.bias, a.bias ? (uint32_t)a.K * 4u : 0u);
    const __amdgpu_buffer_rsrc_t rout = make_rsrc(a.out, a.out_bytes);
    constexpr int ROUNDS = TM / RB, MBR = RB / 32;  // passes, 32-row blocks per pass
#pragma unroll
    for (int rd = 0; rd < ROUNDS; ++rd) {
        if (rd > 0) __syncthreads();
        // the bias values a thread will add (channel-innermost output: its 8 channels are the same for all its vectors)
        // are requested before the exchange through LDS, which covers their latency
        constexpr int CG = RB / 8;
        static_assert(NT % CG == 0, "a thread keeps its channel group over its vectors");
        const int cg = tid % CG;
        const int kv = m0 + rd * RB + cg * 8;
        const bool kok = kv < a.K;  // K % 8 == 0 with that output format: the 8 channels are in or out together
        float bs[8];
        if (onhwc) {
#pragma unroll
            for (int i = 0; i < 8; ++i) bs[i] = buffer_load_elem<float>(rbias, kok ? (uint32_t)(kv + i) * 4u : kOutOfRange);
        }
        // accumulator registers 4i..4i+3 of a lane are rows 8i + 4g .. + 3 of its pixel column: one 16-byte write
#pragma unroll
        for (int mbi = 0; mbi < MBR; ++mbi)
#pragma unroll
            for (int nb = 0; nb < NBW; ++nb) {
                float* dst = &red[(kw * TNP + (wn * NBW + nb) * 32 + li) * RBP + mbi * 32 + 4 * g];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const typename mma_t::acc_t& c = acc[rd * MBR + mbi][nb];
                    *(f32x4*)&dst[8 * i] = f32x4{c[4 * i], c[4 * i + 1], c[4 * i + 2], c[4 * i + 3]};
                }
            }
        if (!onhwc && tid < RB) {
            const int kb = m0 + rd * RB + tid;
            red[KW * TNP * RBP + tid] = buffer_load_elem<float>(rbias, kb < a.K ? (uint32_t)kb * 4u : kOutOfRange);
        }
        __syncthreads();
        if (onhwc) {
            // a thread takes 8 consecutive channels of one pixel: two 16-byte LDS reads per partial sum, one 16-byte store
            constexpr int NV = (CG * TNP + NT - 1) / NT;
            const int k = kv;
#pragma unroll
            for (int j = 0; j < NV; ++j) {
                const int e = j * NT + tid;
                const int col = e / CG, p = p0 + col;
                const bool ok = e < CG * TNP && kok && p < a.P;
                const float* src = &red[(ok ? col : 0) * RBP + cg * 8];
                f32x4 x0 = *(const f32x4*)&src[0], x1 = *(const f32x4*)&src[4];
#pragma unroll
                for (int q = 1; q < KW; ++q) {
                    x0 += *(const f32x4*)&src[q * TNP * RBP];
                    x1 += *(const f32x4*)&src[q * TNP * RBP + 4];
                }
                uint32_t w[4];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    float x = (i < 4 ? x0[i & 3] : x1[i & 3]) + bs[i];
                    if (a.relu) x = x > 0.0f ? x : 0.0f;
                    const uint32_t h = Prec<DT>::from_f32(x);
                    if (i & 1)
                        w[i >> 1] |= h << 16;
                    else
                        w[i >> 1] = h;
                }
                const u32x4 vv = {w[0], w[1], w[2], w[3]};
                __builtin_amdgcn_raw_buffer_store_b128(vv, rout, ok ? (int)((uint32_t)(p * a.K + k) * 2u) : (int)kOutOfRange, 0, 0);
            }
        } else {
            // a thread keeps one pixel and walks down the channels four at a time (16-byte LDS reads); consecutive
            // threads hold consecutive pixels, so each of its 2-byte stores falls into a 128-byte run of one channel
            // plane.  The pixel's image and offset are worked out once; from one group of channels to the next the
            // output offset moves by a constant.
            constexpr int RG = RB / 4;
            constexpr int CPT = NT / TNP > 0 ? NT / TNP : 1;           // channel groups handled side by side
            constexpr int COLS = NT / TNP > 0 ? 1 : (TNP + NT - 1) / NT;  // pixels per thread when the tile is wider than the workgroup
            const float* bsm = &red[KW * TNP * RBP];
#pragma unroll
            for (int cc = 0; cc < COLS; ++cc) {
                const int col = (NT / TNP > 0 ? tid % TNP : tid + cc * NT), rg0 = NT / TNP > 0 ? tid / TNP : 0;
                const int p = p0 + col;
                const bool pok = col < TNP && rg0 < CPT && p < a.P;
                uint32_t n, pix;
                a.dOHW.divmod((uint32_t)(pok ? p : 0), n, pix);
                const int kbase = m0 + rd * RB;
                uint32_t o = (uint32_t)(((int)n * a.K + kbase + rg0 * 4) * a.OHW + (int)pix) * 2u;
                const uint32_t ostep = (uint32_t)a.OHW * 2u;
                const float* src = &red[(pok ? col : 0) * RBP];
#pragma unroll 4
                for (int rg = rg0; rg < RG; rg += CPT) {
                    f32x4 x = *(const f32x4*)&src[rg * 4];
#pragma unroll
                    for (int q = 1; q < KW; ++q) x += *(const f32x4*)&src[q * TNP * RBP + rg * 4];
                    const f32x4 bv = *(const f32x4*)&bsm[rg * 4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        float y = x[i] + bv[i];
                        if (a.relu) y = y > 0.0f ? y : 0.0f;
                        const bool oki = pok && kbase + rg * 4 + i < a.K;
                        buffer_store_elem<elem_t>(Prec<DT>::from_f32(y), rout, oki ? o + (uint32_t)i * ostep : kOutOfRange);
                    }
                    o += 4u * CPT * ostep;
                }
            }
        }
    }
#if PWIN_EXP & 16
    if (tid == 0 && a.ws) tstamp[3] = wall_clock64();
#endif
}

// bytes of the packed filter tensor: K rounded up to whole 32-row blocks
inline size_t packed_filter_bytes(int K, int C, int RS) { return (size_t)((K + 31) / 32) * 32 * (size_t)C * RS * 2; }

template <class CFG>
hipError_t pwin_launch(const Variant&, ConvArgs& a, hipStream_t s)
{
    const hipError_t e = ensure_dynamic_lds((const void*)pwin_kernel<CFG>, CFG::LDS_BYTES);
    if (e != hipSuccess) return e;
    const PwinGeom g = pwin_geom<CFG>(a.N, a.H, a.W, a.K, a.pad, a.OH, a.OW);
    a.dX = make_fastdiv((uint32_t)g.PT);
    a.dY = make_fastdiv((uint32_t)g.PWs);
    a.dZ = make_fastdiv((uint32_t)g.PHs);
    a.filt_bytes = (uint32_t)packed_filter_bytes(a.K, a.C, a.RS);
    hipLaunchKernelGGL(pwin_kernel<CFG>, dim3((unsigned)(g.PT * g.MT)), dim3(CFG::NT), CFG::LDS_BYTES, s, a);
    return hipGetLastError();
}

// The same kernel behind one conversion launch, for layers handed over in the plain formats ([N][C][H][W], [K][C][R][S]):
// the workspace receives the channel-innermost input and the packed filters, the kernel reads those and writes the
// output in the plain format.  Costs a launch and the conversion traffic; pays where the planar window kernels are far
// from the packed kernel's speed (5x5 layers, small batches).
inline size_t pwin_prep_in_bytes(const conv_desc& d) { return (((size_t)d.N * d.C * d.H * d.W * 2) + 255) & ~(size_t)255; }

template <class CFG>
size_t pwin_prep_workspace(const Variant&, const conv_desc& d, int, int)
{
    return pwin_prep_in_bytes(d) + packed_filter_bytes(d.K, d.C, CFG::RS);
}

template <class CFG>
hipError_t pwin_prep_launch(const Variant& v, ConvArgs& a, hipStream_t s)
{
    conv_desc d{};
    d.N = a.N; d.C = a.C; d.H = a.H; d.W = a.W; d.K = a.K;
    unsigned char* ws = (unsigned char*)a.ws;
    void* ws_in = ws;
    void* ws_filt = ws + pwin_prep_in_bytes(d);
    const hipError_t e = launch_prep16(a.in, ws_in, a.N, a.C, a.HW, a.filt, ws_filt, a.K, a.RS, s);
    if (e != hipSuccess) return e;
    ConvArgs b = a;
    b.in = ws_in;
    b.filt = ws_filt;
    return pwin_launch<CFG>(v, b, s);
}

template <class CFG, bool PREP = false>
bool pwin_valid(const Variant&, const conv_desc& d, int OH, int OW)
{
    if (d.dtype != CFG::DT || d.R != CFG::R || d.S != CFG::S || d.stride != 1) return false;
    const uint32_t fmt = d.flags & (CONV_FLAG_IN_NHWC | CONV_FLAG_FILT_KRSC | CONV_FLAG_FILT_PACKED | CONV_FLAG_FILT_WINOGRAD |
                                    CONV_FLAG_OUT_NHWC);
    if (PREP) {
        if (fmt != 0) return false;  // plain formats in and out
    } else if ((fmt & ~CONV_FLAG_OUT_NHWC) != (CONV_FLAG_IN_NHWC | CONV_FLAG_FILT_PACKED)) {
        return false;
    }
    if (d.flags & CONV_FLAG_MAXPOOL_3X3S2) return false;
    if ((d.C % CFG::CB) != 0) return false;
    if ((d.flags & CONV_FLAG_OUT_NHWC) && (d.K % 8) != 0) return false;
    // shared borders hold every out-of-image tap only while the border is no wider than the window's reach
    if (d.pad > CFG::R - 1 || d.pad > CFG::S - 1) return false;
    const PwinGeom g = pwin_geom<CFG>(d.N, d.H, d.W, d.K, d.pad, OH, OW);
    if (g.span > CFG::SLOTS) return false;
    if ((long long)g.PT * g.MT > 0x7fffffffLL) return false;
    const long long lim = 1LL << 31;  // byte offsets are formed in 32 bits with room for the look-ahead past the end
    if ((long long)d.N * d.C * d.H * d.W * 2 >= lim || (long long)packed_filter_bytes(d.K, d.C, CFG::RS) >= lim) return false;
    if ((long long)d.N * d.K * OH * OW * 2 >= lim) return false;
    return true;
}

template <class CFG>
void pwin_register(std::vector<Variant>& out)
{
    Variant v;
    char buf[160];
    // (the 32-row tiles for small operations come with several slab sizes: theirs is part of the name)
    char slots[24] = "";
    if (CFG::TM == 32) snprintf(slots, sizeof slots, "_s%d", CFG::SLOTS);
    snprintf(buf, sizeof buf, "pwin_%s_%dx%d_M%dN%dC%d_w%dx%d_a%d%s%s", dtype_name(CFG::DT), CFG::R, CFG::S, CFG::TM, CFG::TNP,
             CFG::CB, CFG::KW, CFG::WN, CFG::AD, CFG::ALIGN8 ? "_p8" : "", slots);
    v.name = buf;
    v.dtype = CFG::DT;
    v.split = 1;
    v.tm = CFG::TM;
    v.tn = CFG::TNP;
    v.tk = CFG::CB * CFG::RS;
    v.threads = CFG::NT;
    v.family = FAM_NHWC;
    v.specificity = 6;
    v.traits = TRAIT_PACKED_FILTERS;
    v.valid = &pwin_valid<CFG>;
    v.launch = &pwin_launch<CFG>;
    out.push_back(v);
    // the twin for the plain formats: one conversion launch into the workspace, then the same kernel
    v.name += "_prep";
    v.family = FAM_WINDOW;
    v.specificity = 4;
    v.traits = TRAIT_CONVERTS_FIRST;
    v.valid = &pwin_valid<CFG, true>;
    v.launch = &pwin_prep_launch<CFG>;
    v.ws_extra = &pwin_prep_workspace<CFG>;
    out.push_back(v);
}

}  // namespace convfwd
