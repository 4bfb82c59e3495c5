// Window-reuse convolution for stride-1 layers in fp32 on the plain formats ([N][C][H][W], [K][C][R][S]) with the
// reduction split over the waves of a workgroup -- the fp32 counterpart of the packed-filter kernel's organisation.
//
// What it is for: the 3x3 / 5x5 layers of the benchmark set at small batch have a few hundred 32x32 output blocks for
// 1024 SIMDs.  The older kernels filled the chip by splitting the reduction over workgroups and paid a second launch
// for the sum; here KW = 4 / 8 / 16 waves of ONE workgroup split the channels of a chunk, every wave multiplies its
// channels for the whole output tile, and the partial tiles meet in LDS at the end (added in wave order:
// deterministic), so a layer with 72 output blocks still runs as one launch of 72 x 16 waves.
//   * Pixel axis linear over (image, row, column); the input slab in LDS is [channel][position] over the stack of all
//     images with shared zero borders (row pitch W + pad, image pitch H + pad rows), as in pwin_kernel.h: the operand
//     of pixel p at tap (r,s) is slab[c][base(p) + r*(W+pad) + s] whatever image p belongs to.  fp32 MFMA 32x32x2 takes
//     one value per lane with lane half h supplying reduction index h: half h reads channel 2i + h of the wave's
//     channels, so both halves use the same tap offset and no index arithmetic depends on the lane half.
//   * The filter slab of a chunk is [TM][CB*R*S]: contiguous pieces of KCRS rows, copied with 16-byte loads (no
//     repacking of the filters: this is the plain contract); a lane's filter value for (channel, tap) is one LDS read.
//   * Next chunk's global loads are issued at the start of a chunk and written to the other LDS buffer in the middle
//     of it; one barrier per chunk, before its last tap.
#pragma once

#include "pwin_kernel.h"

// Compile-time experiment hook (0 in the product): bit 16 = workgroups write phase time stamps (100 MHz ticks) into the
// workspace, 8 per workgroup, when one is passed.
#ifndef PWIN32_EXP
#define PWIN32_EXP 0
#endif
#if PWIN32_EXP & 16
#define PWIN32_STAMP(i) do { if (tid == 0 && a.ws) ((unsigned long long*)a.ws)[(size_t)blockIdx.x * 8 + (i)] = wall_clock64(); } while (0)
#else
#define PWIN32_STAMP(i) do { } while (0)
#endif

namespace convfwd {

template <int R_, int S_, int KW_, int WN_, int TMB_, int NBW_, int CPW_, int SLOTS_, int PD_ = 1>
struct Pwin32Cfg {
    static constexpr int R = R_, S = S_, KW = KW_, WN = WN_, TMB = TMB_, NBW = NBW_, CPW = CPW_, SLOTS = SLOTS_;
    // PD: how many steps ahead of its MFMAs a step's operands are read from LDS (PD + 1 register sets).  A step of a
    // 32 x 32 wave tile is ONE 64-cycle MFMA, less than an LDS round trip: small tiles read two or more steps ahead.
    static constexpr int PD = PD_, SETS = PD_ + 1;
    static_assert(((CPW_ / 2) * R_ * S_) % (PD_ + 1) == 0, "the register sets must divide the steps of a chunk");
    static_assert(CPW % 2 == 0, "a wave takes its channels in pairs (one per lane half)");
    static constexpr int RS = R * S;
    static constexpr int NT = 64 * KW * WN;
    static_assert(NT <= 1024, "workgroup size");
    static constexpr int CB = CPW * KW;          // channels per chunk
    static constexpr int TM = 32 * TMB, TNP = 32 * NBW * WN;
    static constexpr int KCH = CB * RS;          // filter elements per row and chunk
    static_assert(KCH % 4 == 0, "filter slab rows are moved as 16-byte vectors");
    static constexpr int LDA = KCH + 4;          // filter slab row pitch (floats; rows stay 16-byte aligned)
    static constexpr int A_VECS = TM * KCH / 4;
    static constexpr int LBA = (A_VECS + NT - 1) / NT;  // filter vectors per thread
    static constexpr int SP = SLOTS + 32;        // channel pitch of the input slab: the two lane halves read 32 banks apart
    static constexpr int B_ELEMS = CB * SLOTS;
    static_assert(B_ELEMS % NT == 0, "every thread stages the same number of input values");
    static constexpr int LBT = B_ELEMS / NT;
    static constexpr int BUF_FLOATS = TM * LDA + CB * SP;
    static constexpr int RB = ((size_t)KW * TNP * (TM + 4) * 4 + TM * 4 <= 160 * 1024) ? TM : 32;
    static constexpr int RBP = RB + 4;
    static constexpr size_t LDS_PIPE = sizeof(float) * 2 * (size_t)BUF_FLOATS;
    static constexpr size_t LDS_RED = sizeof(float) * ((size_t)KW * TNP * RBP + RB);
    static constexpr size_t LDS_BYTES = LDS_PIPE > LDS_RED ? LDS_PIPE : LDS_RED;
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
};

template <class CFG>
inline PwinGeom pwin32_geom(int N, int H, int W, int K, int pad, int OH, int OW)
{
    PwinGeom g;
    g.PWs = W + pad;
    g.PHs = H + pad;
    const long long P = (long long)N * OH * OW;
    g.PT = (int)((P + CFG::TNP - 1) / CFG::TNP);
    g.MT = (K + CFG::TM - 1) / CFG::TM;
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
__global__ __launch_bounds__(CFG::NT) void pwin32_kernel(ConvArgs a)
{
    constexpr int R = CFG::R, S = CFG::S, RS = CFG::RS, KW = CFG::KW, WN = CFG::WN, TMB = CFG::TMB, NBW = CFG::NBW;
    constexpr int CPW = CFG::CPW, SLOTS = CFG::SLOTS, NT = CFG::NT, CB = CFG::CB, TM = CFG::TM, TNP = CFG::TNP, KCH = CFG::KCH;
    constexpr int LDA = CFG::LDA, A_VECS = CFG::A_VECS, LBA = CFG::LBA, SP = CFG::SP, LBT = CFG::LBT, BUF = CFG::BUF_FLOATS;
    constexpr int RB = CFG::RB, RBP = CFG::RBP, PD = CFG::PD, SETS = CFG::SETS;
    typedef Mma<CONV_F32, 32> mma_t;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    float* const buf0 = (float*)smem_raw;  // [2][ filter slab TM*LDA | input slab CB*SP ]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kw = wave % KW, wn = wave / KW;
    const int li = lane & 31, h = lane >> 5;
    PWIN32_STAMP(0);

    const int PT = (int)a.dX.d, PWs = (int)a.dY.d, PHs = (int)a.dZ.d;
    const int MT = (a.K + TM - 1) / TM, T = MT * PT;
    int logical;
    {
        const int b = blockIdx.x, x = b & 7, q = b >> 3;
        const int per = T >> 3, rem = T & 7;
        logical = x * per + (x < rem ? x : rem) + q;
    }
    uint32_t mt_u, pt_u;
    a.dX.divmod((uint32_t)logical, mt_u, pt_u);
    const int m0 = (int)mt_u * TM, p0 = (int)pt_u * TNP;
    const int plast = (p0 + TNP < a.P ? p0 + TNP : a.P) - 1;
    auto base_pos = [&](int p) {
        uint32_t n, pix, oy, ox;
        a.dOHW.divmod((uint32_t)p, n, pix);
        a.dOW.divmod(pix, oy, ox);
        return ((int)n * PHs + (int)oy) * PWs + (int)ox;
    };
    const int lo = base_pos(p0);
    const int nposw = base_pos(plast) + (R - 1) * PWs + S - lo;

    const __amdgpu_buffer_rsrc_t rin = make_rsrc(a.in, a.in_bytes);
    const __amdgpu_buffer_rsrc_t rfilt = make_rsrc(a.filt, a.filt_bytes);

    // ---- staging plans (chunk independent; a chunk adds its channel offset) ----------------------------------------
    // filter slab: vector v = (row v / (KCH/4), 16-byte vector v % (KCH/4) of the row's chunk piece)
    uint32_t f_goff[LBA];
#pragma unroll
    for (int i = 0; i < LBA; ++i) {
        const int v = i * NT + tid;
        const int row = v / (KCH / 4), q4 = v % (KCH / 4);
        const bool ok = v < A_VECS && m0 + row < a.K;
        f_goff[i] = ok ? (uint32_t)((m0 + row) * a.C * RS + q4 * 4) * 4u : kOutOfRange;
    }
    // input slab: value t = (channel t / SLOTS of the chunk, position t % SLOTS)
    uint32_t t_goff[LBT];
#pragma unroll
    for (int i = 0; i < LBT; ++i) {
        const int t = i * NT + tid;
        const int ch = t / SLOTS, j = t % SLOTS;
        uint32_t Y, X, n, yy;
        a.dY.divmod((uint32_t)(lo + j), Y, X);
        a.dZ.divmod(Y, n, yy);
        const bool ok = j < nposw && (int)X >= a.pad && (int)X < a.pad + a.W && (int)yy >= a.pad && (int)n < a.N;
        t_goff[i] = ok ? (uint32_t)((((int)n * a.C + ch) * a.H + (int)yy - a.pad) * a.W + (int)X - a.pad) * 4u : kOutOfRange;
    }
    uint4 a_reg[LBA];
    float b_reg[LBT];
    const uint32_t f_step = (uint32_t)KCH * 4u, b_step = (uint32_t)CB * (uint32_t)a.HW * 4u;
    auto load_chunk = [&](int chunk) {
        const uint32_t fo = (uint32_t)chunk * f_step, bo = (uint32_t)chunk * b_step;
#pragma unroll
        for (int i = 0; i < LBA; ++i) a_reg[i] = buffer_load_vec(rfilt, f_goff[i] == kOutOfRange ? kOutOfRange : f_goff[i] + fo);
#pragma unroll
        for (int i = 0; i < LBT; ++i) b_reg[i] = buffer_load_elem<float>(rin, t_goff[i] == kOutOfRange ? kOutOfRange : t_goff[i] + bo);
    };
    auto store_chunk = [&](int buf) {
        float* As = buf0 + buf * BUF;
        float* Bs = As + TM * LDA;
#pragma unroll
        for (int i = 0; i < LBA; ++i) {
            const int v = i * NT + tid;
            if (LBA * NT == A_VECS || v < A_VECS) *(uint4*)&As[(v / (KCH / 4)) * LDA + (v % (KCH / 4)) * 4] = a_reg[i];
        }
#pragma unroll
        for (int i = 0; i < LBT; ++i) {
            const int t = i * NT + tid;
            Bs[(t / SLOTS) * SP + (t % SLOTS)] = b_reg[i];
        }
    };

    // per lane: filter row and channel of its half inside the wave's channels; window origin of each pixel column
    const int a_lane = li * LDA + (kw * CPW + h) * RS;       // + mb*32*LDA + pair*2*RS + tap
    int bpos[NBW];
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb) {
        const int p = p0 + (wn * NBW + nb) * 32 + li;
        bpos[nb] = (kw * CPW + h) * SP + base_pos(p < a.P ? p : plast) - lo;  // + pair*2*SP + r*PWs + s
    }

    typename mma_t::acc_t acc[TMB][NBW];
#pragma unroll
    for (int mb = 0; mb < TMB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mb][nb][v] = 0.0f;

    const int nchunks = a.C / CB;
    PWIN32_STAMP(1);
    load_chunk(0);
    store_chunk(0);
    load_chunk(1);  // unconditional: with a single chunk the data is never used
    __syncthreads();
    PWIN32_STAMP(2);

    constexpr int STEPS = (CPW / 2) * RS;  // MFMA steps of a wave per chunk: (channel pair, tap)
    float af[SETS][TMB], bf[SETS][NBW];
    auto read_step = [&](const float* As, const float* Bs, int step, int set) {
        const int pair = step / RS, t = step % RS, r = t / S, s = t % S;
#pragma unroll
        for (int mb = 0; mb < TMB; ++mb) af[set][mb] = As[a_lane + mb * 32 * LDA + pair * 2 * RS + t];
        const int toff = pair * 2 * SP + r * PWs + s;
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb) bf[set][nb] = Bs[bpos[nb] + toff];
    };
    static_for<PD>([&](auto ic) { read_step(buf0, buf0 + TM * LDA, decltype(ic)::value, decltype(ic)::value); });

    constexpr int TSTORE = (STEPS - PD) / 2;
    int buf = 0;
    auto do_chunk = [&](auto store_c, auto load_c, int chunk) {
        constexpr bool STORE = decltype(store_c)::value, LOAD = decltype(load_c)::value;
        const float* As = buf0 + buf * BUF;
        const float* Bs = As + TM * LDA;
        const float* An = buf0 + (buf ^ 1) * BUF;
        const float* Bn = An + TM * LDA;
        static_for<STEPS>([&](auto tc) {
            constexpr int t = decltype(tc)::value, cur = t % SETS, nxt = (t + PD) % SETS;
            // every wave has read the last operands it takes from this chunk's buffer: the other buffer (stored at step
            // TSTORE by everyone) becomes readable; after the last chunk the reduction buffer may overlay the slabs
            if constexpr (t == STEPS - PD) __syncthreads();
            if constexpr (t + PD < STEPS) {
                read_step(As, Bs, t + PD, nxt);
            } else if constexpr (STORE) {
                read_step(An, Bn, t + PD - STEPS, nxt);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int mb = 0; mb < TMB; ++mb)
#pragma unroll
                for (int nb = 0; nb < NBW; ++nb) acc[mb][nb] = mma_t::run(af[cur][mb], bf[cur][nb], acc[mb][nb]);
            if constexpr (t == TSTORE) {
                if constexpr (STORE) store_chunk(buf ^ 1);
                if constexpr (LOAD) load_chunk(chunk + 2);
            }
            __builtin_amdgcn_sched_barrier(0);
        });
        buf ^= 1;
    };
    {
        int chunk = 0;
        for (; chunk + 2 < nchunks; ++chunk) do_chunk(std::true_type{}, std::true_type{}, chunk);
        if (chunk + 1 < nchunks) do_chunk(std::true_type{}, std::false_type{}, chunk++);
        do_chunk(std::false_type{}, std::false_type{}, chunk);
    }

    PWIN32_STAMP(3);
    // ---- add the KW channel-waves' partial sums in wave order, then bias + activation + store ----------------------
    float* const red = (float*)smem_raw;  // [KW][TNP][RBP] + [RB] bias
    const __amdgpu_buffer_rsrc_t rbias = make_rsrc(a.bias, a.bias ? (uint32_t)a.K * 4u : 0u);
    const __amdgpu_buffer_rsrc_t rout = make_rsrc(a.out, a.out_bytes);
    constexpr int ROUNDS = TM / RB, MBR = RB / 32;
#pragma unroll
    for (int rd = 0; rd < ROUNDS; ++rd) {
        if (rd > 0) __syncthreads();
#pragma unroll
        for (int mbi = 0; mbi < MBR; ++mbi)
#pragma unroll
            for (int nb = 0; nb < NBW; ++nb) {
                float* dst = &red[(kw * TNP + (wn * NBW + nb) * 32 + li) * RBP + mbi * 32 + 4 * h];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const typename mma_t::acc_t& c = acc[rd * MBR + mbi][nb];
                    *(f32x4*)&dst[8 * i] = f32x4{c[4 * i], c[4 * i + 1], c[4 * i + 2], c[4 * i + 3]};
                }
            }
        if (tid < RB) {
            const int kb = m0 + rd * RB + tid;
            red[KW * TNP * RBP + tid] = buffer_load_elem<float>(rbias, kb < a.K ? (uint32_t)kb * 4u : kOutOfRange);
        }
        __syncthreads();
        // a thread keeps one pixel and walks down the channels four at a time; consecutive threads, consecutive pixels
        constexpr int RG = RB / 4;
        constexpr int CPT = NT / TNP > 0 ? NT / TNP : 1;
        constexpr int COLS = NT / TNP > 0 ? 1 : (TNP + NT - 1) / NT;
        const float* bsm = &red[KW * TNP * RBP];
        const uint32_t ostep = (uint32_t)a.OHW * 4u;
#pragma unroll
        for (int cc = 0; cc < COLS; ++cc) {
            const int col = (NT / TNP > 0 ? tid % TNP : tid + cc * NT), rg0 = NT / TNP > 0 ? tid / TNP : 0;
            const int p = p0 + col;
            const bool pok = col < TNP && rg0 < CPT && p < a.P;
            uint32_t n, pix;
            a.dOHW.divmod((uint32_t)(pok ? p : 0), n, pix);
            const int kbase = m0 + rd * RB;
            uint32_t o = (uint32_t)(((int)n * a.K + kbase + rg0 * 4) * a.OHW + (int)pix) * 4u;
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
                    buffer_store_elem<float>(y, rout, oki ? o + (uint32_t)i * ostep : kOutOfRange);
                }
                o += 4u * CPT * ostep;
            }
        }
    }
    PWIN32_STAMP(4);
}

template <class CFG>
hipError_t pwin32_launch(const Variant&, ConvArgs& a, hipStream_t s)
{
    const hipError_t e = ensure_dynamic_lds((const void*)pwin32_kernel<CFG>, CFG::LDS_BYTES);
    if (e != hipSuccess) return e;
    const PwinGeom g = pwin32_geom<CFG>(a.N, a.H, a.W, a.K, a.pad, a.OH, a.OW);
    a.dX = make_fastdiv((uint32_t)g.PT);
    a.dY = make_fastdiv((uint32_t)g.PWs);
    a.dZ = make_fastdiv((uint32_t)g.PHs);
    hipLaunchKernelGGL(pwin32_kernel<CFG>, dim3((unsigned)(g.PT * g.MT)), dim3(CFG::NT), CFG::LDS_BYTES, s, a);
    return hipGetLastError();
}

template <class CFG>
bool pwin32_valid(const Variant&, const conv_desc& d, int OH, int OW)
{
    if (d.dtype != CONV_F32 || d.R != CFG::R || d.S != CFG::S || d.stride != 1) return false;
    if (d.flags & ~(uint32_t)CONV_FLAG_RELU) return false;  // plain formats, no fused pool
    if ((d.C % CFG::CB) != 0) return false;
    if (d.pad > CFG::R - 1 || d.pad > CFG::S - 1) return false;
    const PwinGeom g = pwin32_geom<CFG>(d.N, d.H, d.W, d.K, d.pad, OH, OW);
    if (g.span > CFG::SLOTS) return false;
    if ((long long)g.PT * g.MT > 0x7fffffffLL) return false;
    const long long lim = 1LL << 31;
    if ((long long)d.N * d.C * d.H * d.W * 4 >= lim || (long long)d.K * d.C * CFG::RS * 4 >= lim) return false;
    if ((long long)d.N * d.K * OH * OW * 4 >= lim) return false;
    return true;
}

template <class CFG>
void pwin32_register(std::vector<Variant>& out)
{
    Variant v;
    char buf[160];
    snprintf(buf, sizeof buf, "pwin_f32_%dx%d_M%dN%dC%d_w%dx%d_s%d_d%d", CFG::R, CFG::S, CFG::TM, CFG::TNP, CFG::CB, CFG::KW, CFG::WN,
             CFG::SLOTS, CFG::PD);
    v.name = buf;
    v.dtype = CONV_F32;
    v.split = 1;
    v.tm = CFG::TM;
    v.tn = CFG::TNP;
    v.tk = CFG::CB * CFG::RS;
    v.threads = CFG::NT;
    v.family = FAM_WINDOW;
    v.specificity = 5;
    v.traits = TRAIT_CHANNEL_WAVES;
    v.valid = &pwin32_valid<CFG>;
    v.launch = &pwin32_launch<CFG>;
    out.push_back(v);
}

}  // namespace convfwd
