// Window-reuse convolution for strided layers with very few input channels (the first layer of a network: 11x11
// stride 4 or 7x7 stride 2 over 3 channels), fp16 / bf16 storage, 32x32x16 MFMA with fp32 accumulation.
//
// What the gather kernels pay for on these layers is the im2col expansion itself: with R*S = 121 taps every input
// element is fetched dozens of times, two bytes at a time, and the loop waits on those fetches.  Here the input rows a
// tile of output pixels touches are copied into LDS once (paper, Section 5 "Related Work": overlapping windows share
// the copy) and every operand is an LDS read:
//   * the reduction runs over (filter row, channel, group of 4 taps): a filter row of S taps is padded to 4*SQ, so a
//     lane's 8 reduction elements of one MFMA are two groups, each 4 consecutive input columns of one input row,
//     ST*ox + 4*g .. +3: contiguous in the staged row and aligned (8 bytes for stride 4, 4 bytes for stride 2);
//   * the filters are re-laid once per workgroup into [TM][KP] with zeros in the padding taps and stay in LDS;
//     the patch operand's padding taps are cleared as well, so a non-finite input value reaches only the outputs
//     whose window holds it;
//   * a tile is 128 consecutive output pixels of one image (any row length: a tile may span several output rows),
//     one 32-pixel block per wave, all TM channels per wave.  The workgroup is persistent and made of two groups of 4
//     waves, each walking over its own tiles in its own patch buffer (a second wave per SIMD to issue while the first
//     waits): a group fetches the rows of its next tile while it multiplies; the filters are staged once, by all waves;
//   * zero padding and rows or columns past the image are zero elements of the staged rows.
#pragma once

#include "ugemm_kernel.h"

namespace convfwd {

typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

struct u32x3 {  // what a 12-byte buffer load returns (the vector type is padded to 16 bytes)
    uint32_t x, y, z, unused;
};

template <int DT_, int C_, int R_, int S_, int ST_, int TMB_, int IRMAX_, int PITCH_>
struct Swin16Cfg {
    static_assert(DT_ == CONV_F16 || DT_ == CONV_BF16, "16-bit storage only");
    static_assert(ST_ == 2 || ST_ == 4, "operand groups must stay dword aligned");
    static_assert(PITCH_ % 4 == 0, "staged rows keep the groups' alignment");
    static constexpr int DT = DT_, C = C_, R = R_, S = S_, ST = ST_, TMB = TMB_, IRMAX = IRMAX_, PITCH = PITCH_;
    static constexpr int CWAVES = 4;                 // waves of a group: one 32-pixel block each
    static constexpr int NBW = 1;
    static constexpr int WAVES = 8, NT = 64 * WAVES; // two groups, each on its own tile and patch buffer; all waves re-lay the filters
    static constexpr int TM = 32 * TMB;              // output channels per workgroup
    static constexpr int TN = 32 * CWAVES;           // pixels per tile
    static constexpr int SQ = (S + 3) / 4;           // groups of 4 taps per filter row
    static constexpr int NROW = C * R;               // (filter row, channel) pairs: "lines" of the reduction
    static constexpr int NPAIR = (NROW + 1) / 2;     // the two lane halves of an MFMA take the lines 2t and 2t+1
    static constexpr int KSTEPS = (NPAIR * SQ + 1) / 2;  // MFMA steps: two groups per lane half
    static constexpr int KP = KSTEPS * 16;           // padded reduction length
    static constexpr int LDA = KP + 8;               // filter row pitch: rows 16-byte aligned, conflict-free 16-byte reads
    static constexpr int SROWS = C * IRMAX;          // staged rows of one tile, [input row][channel]
    static constexpr int RR_W = (IRMAX + CWAVES - 1) / CWAVES;  // input rows per wave (each in all C channels)
    static constexpr int ROWS_W = RR_W * C;          // staged rows per wave
    static constexpr int B_ELEMS = (SROWS + 1) * PITCH;  // one patch buffer; the last row stays zero
};

// output rows a tile of TN consecutive pixels can touch
inline int swin16_rows_spanned(int OH, int OW, int TN)
{
    int rows = (TN - 1 + OW - 1) / OW + 1;
    return rows < OH ? rows : OH;
}

// ---- filters: KCRS rows -> LDS [TM][KP] (+ the tile's biases) -----------------------------------------------------
// Reduction element kk = 16*j + 8*half + 4*g + e of MFMA step j belongs to line 2t + half (line = r*C + c) and tap
// 4*sq + e, where (t, sq) = divmod(2j + g, SQ); lines and taps that do not exist are zeros.  A thread owns one group
// slot (4 taps, 8 bytes of LDS) and walks down the filter rows, NT/128 at a time per workgroup.  The caller's barrier
// publishes the result.
template <class CFG>
__device__ __forceinline__ void swin16_stage_filters(uint16_t* As, float* bias_s, __amdgpu_buffer_rsrc_t rfilt, const ConvArgs& a,
                                                     int m0, int tid)
{
    constexpr int C = CFG::C, R = CFG::R, S = CFG::S, SQ = CFG::SQ, NROW = CFG::NROW, KP = CFG::KP, LDA = CFG::LDA;
    constexpr int TM = CFG::TM, NT = CFG::NT, Q = C * R * S;
    static_assert(S % 4 == 0 || S % 4 == 3, "a filter row's last group holds 3 or 4 taps");
    constexpr int GS = KP / 4;
    static_assert(GS <= 128, "a filter row's groups fit 128 threads");
    constexpr int MR = NT / 128;  // filter rows per pass of the workgroup (even: a thread's rows keep their parity)
    static_assert(NT % 128 == 0 && MR % 2 == 0, "rows per pass");
    const int gs = tid & 127, mrow = __builtin_amdgcn_readfirstlane(tid >> 7);
    const int j = gs >> 2, gh = (gs >> 1) & 1, g = gs & 1;
    const int i2 = 2 * j + g, t = i2 / SQ, sq = i2 - t * SQ;
    const int line = 2 * t + gh;
    const int fr = line / C, fc = line - fr * C;
    const bool g_ok = gs < GS && line < NROW;
    const int src = (fc * R + fr) * S + 4 * sq;                 // first tap of the group in the filter row
    const bool three = S - 4 * sq < 4;
    // The group's 8 bytes start at element m*Q + src, even or odd: they are cut out of three aligned dwords (a
    // misaligned dword load runs at a fraction of the rate).  The rows of a thread are MR apart, so m*Q keeps its
    // parity pm and the cut is the same for every row: vector part 2*((src+pm) & ~1), scalar part 2*(m*Q & ~1).
    const int pm = ((m0 + mrow) * Q) & 1;
    const int par = (pm + src) & 1;
    const uint32_t v0 = g_ok ? (uint32_t)((src + pm) & ~1) * 2u : kFarOffset;
    constexpr int NIT = (TM + MR - 1) / MR;
    // the last pass may reach past the tile's rows when MR does not divide TM (decided at compile time otherwise)
    auto row_in = [&](int it) { return TM % MR == 0 || MR * it + MR <= TM || mrow + MR * it < TM; };
    u32x3 f[NIT];
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int m = m0 + mrow + MR * it;
        const uint32_t soff = (m < a.K && row_in(it)) ? (uint32_t)((m * Q) & ~1) * 2u : kFarScalar;
        f[it] = __builtin_bit_cast(u32x3, __builtin_amdgcn_raw_buffer_load_b96(rfilt, (int)v0, (int)soff, 0));
    }
    if (tid < TM) {
        const __amdgpu_buffer_rsrc_t rbias = make_rsrc(a.bias, a.bias ? (uint32_t)a.K * 4u : 0u);
        bias_s[tid] = buffer_load_elem<float>(rbias, m0 + tid < a.K ? (uint32_t)(m0 + tid) * 4u : kOutOfRange);
    }
    if (gs < GS) {
        const uint32_t sh = par ? 16u : 0u, mhi = three ? 0x0000FFFFu : 0xFFFFFFFFu;
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const uint32_t lo = __builtin_amdgcn_alignbit(f[it].y, f[it].x, sh);
            const uint32_t hi = __builtin_amdgcn_alignbit(f[it].z, f[it].y, sh);
            if (row_in(it)) *(uint2*)&As[(mrow + MR * it) * LDA + 4 * gs] = make_uint2(lo, hi & mhi);
        }
    }
}

// ---- the reduction of a wave's NBW 32-pixel blocks: acc[mb][nb] += filters[mb*32 + ..][:] * window_nb[:] -----------------
// Ap: the lane's filter row and half (As + li*LDA + 8*h); Bp[nb]: the first element of the lane's window of block nb in
// line h (staged row (window's first input row)*C + h, column ST * ox).  Operands of step j+1 are read while step j
// multiplies; a filter fragment serves NBW products, a window fragment TMB.
template <class CFG>
__device__ __forceinline__ void swin16_mma_loop(const uint16_t* __restrict__ Ap, const uint16_t* const (&Bp)[CFG::NBW],
                                                uint32_t last_pair_mask,
                                                typename Mma<CFG::DT, 32>::acc_t (&acc)[CFG::TMB][CFG::NBW])
{
    constexpr int S = CFG::S, ST = CFG::ST, TMB = CFG::TMB, NBW = CFG::NBW, PITCH = CFG::PITCH, SQ = CFG::SQ, NROW = CFG::NROW;
    constexpr int KSTEPS = CFG::KSTEPS, LDA = CFG::LDA;
    typedef Mma<CFG::DT, 32> mma_t;
    uint4 af[2][TMB], bf[2][NBW];
    auto read_step = [&](int j, int slot) {
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb) {
            uint32_t bw[4];
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                const int i2 = 2 * j + g, t = i2 / SQ, sq = i2 % SQ;
                // compile-time, an immediate offset of the read; slots past the last line read the window's start
                const int off = 2 * t >= NROW ? 0 : 2 * t * PITCH + 4 * sq;
                uint32_t lo, hi;
                if constexpr (ST % 4 == 0) {
                    const uint2 w = *(const uint2*)&Bp[nb][off];
                    lo = w.x;
                    hi = w.y;
                } else {
                    const uint32_t* w = (const uint32_t*)&Bp[nb][off];
                    lo = w[0];
                    hi = w[1];
                }
                bw[2 * g] = lo;
                bw[2 * g + 1] = hi;
            }
            bf[slot][nb] = make_uint4(bw[0], bw[1], bw[2], bw[3]);
        }
#pragma unroll
        for (int mb = 0; mb < TMB; ++mb) af[slot][mb] = *(const uint4*)&Ap[mb * 32 * LDA + 16 * j];
    };
    read_step(0, 0);
#pragma unroll
    for (int j = 0; j < KSTEPS; ++j) {
        if (j + 1 < KSTEPS) read_step(j + 1, (j + 1) & 1);
        __builtin_amdgcn_sched_barrier(0);  // keep the reads ahead of the products they overlap with
        // padding taps and lines that do not exist are cleared here, one step after their read was issued
        uint4 b[NBW];
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb) {
            b[nb] = bf[j & 1][nb];
            uint32_t* bw = (uint32_t*)&b[nb];
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                const int i2 = 2 * j + g, t = i2 / SQ, sq = i2 % SQ;
                const int ntap = 2 * t >= NROW ? 0 : (S - 4 * sq >= 4 ? 4 : S - 4 * sq);
                // (asm: a plain AND has no tie to this point of the program and is moved up to its read, where it waits;
                // the s_nop is the gap the hardware needs between a VALU write and an MFMA reading the register, which the
                // compiler does not insert after inline assembly)
                if (ntap < 2) asm volatile("v_and_b32 %0, %1, %0\n\ts_nop 1" : "+v"(bw[2 * g]) : "v"(ntap == 1 ? 0x0000FFFFu : 0u));
                if (ntap < 4) asm volatile("v_and_b32 %0, %1, %0\n\ts_nop 1" : "+v"(bw[2 * g + 1]) : "v"(ntap == 3 ? 0x0000FFFFu : 0u));
                if (2 * t + 1 >= NROW) {
                    asm volatile("v_and_b32 %0, %1, %0\n\ts_nop 1" : "+v"(bw[2 * g]) : "v"(last_pair_mask));
                    asm volatile("v_and_b32 %0, %1, %0\n\ts_nop 1" : "+v"(bw[2 * g + 1]) : "v"(last_pair_mask));
                }
            }
        }
#pragma unroll
        for (int mb = 0; mb < TMB; ++mb)
#pragma unroll
            for (int nb = 0; nb < NBW; ++nb) acc[mb][nb] = mma_t::run(af[j & 1][mb], b[nb], acc[mb][nb]);
        __builtin_amdgcn_sched_barrier(0);
    }
}

template <class CFG>
__global__ __launch_bounds__(CFG::NT) void swin16_kernel(ConvArgs a)
{
    typedef uint16_t elem_t;
    constexpr int DT = CFG::DT, C = CFG::C, R = CFG::R, S = CFG::S, ST = CFG::ST, TMB = CFG::TMB, PITCH = CFG::PITCH;
    constexpr int NT = CFG::NT, WAVES = CFG::CWAVES, TM = CFG::TM, TN = CFG::TN, SQ = CFG::SQ, NROW = CFG::NROW;
    constexpr int KSTEPS = CFG::KSTEPS, KP = CFG::KP, LDA = CFG::LDA, ROWS_W = CFG::ROWS_W, RR_W = CFG::RR_W, IRMAX = CFG::IRMAX;
    constexpr int SROWS = CFG::SROWS, B_ELEMS = CFG::B_ELEMS, Q = C * R * S;
    typedef Mma<DT, 32> mma_t;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];

    elem_t* const As = (elem_t*)smem_raw;          // [TM][LDA]
    elem_t* const Bs0 = As + TM * LDA;             // [2][B_ELEMS]
    float* const bias_s = (float*)(Bs0 + 2 * B_ELEMS);  // [TM]

    const int tid = threadIdx.x, lane = tid & 63;
    const int grp = __builtin_amdgcn_readfirstlane(tid >> 8);        // wave group: tiles t_begin + grp, + 2, ... in patch buffer grp
    const int wave = __builtin_amdgcn_readfirstlane((tid >> 6) & 3);  // wave of the group
    const int li = lane & 31, h = lane >> 5;
    const int m0 = blockIdx.y * TM;
    const int tiles = a.N * (int)a.dX.d;           // dX divides by the tiles of one image
    // Workgroups are dealt to the 8 XCDs in turn, each XCD with its own L2: workgroup -> logical id such that an XCD
    // gets one contiguous run of ids, and a logical id one contiguous run of tiles.  Neighbouring tiles share input
    // rows, so each XCD fetches its images once instead of every XCD fetching every image.
    int t_begin, t_end;
    {
        const int G = (int)gridDim.x, per = (G + 7) / 8, rem = G % 8;
        const int x = (int)blockIdx.x % 8, y = (int)blockIdx.x / 8;
        const int lid = (rem == 0 || x < rem) ? x * per + y : rem * per + (x - rem) * (per - 1) + y;
        const int tpw = (tiles + G - 1) / G;
        t_begin = lid * tpw;
        t_end = t_begin + tpw < tiles ? t_begin + tpw : tiles;
    }

    // whole dwords: the tensors' last elements may be the low halves of aligned dwords
    const __amdgpu_buffer_rsrc_t rin = make_rsrc(a.in, (a.in_bytes + 3u) & ~3u);
    const __amdgpu_buffer_rsrc_t rfilt = make_rsrc(a.filt, (a.filt_bytes + 3u) & ~3u);

    // ---- input rows of a tile -> registers -> LDS -------------------------------------------------------------
    // staged row rr*C + c holds input row iy_first + rr of channel c, staged column x holds input column x - pad.
    // A lane covers 4 columns (8 bytes) of a row (PITCH = 256 columns).  A row starts
    // at any 2-byte alignment in memory, and a misaligned load runs at a fraction of the rate: the two dwords are
    // fetched from the aligned address at or one element before the row's origin, and in the second case shifted by
    // one element when they go to LDS (the missing half comes from the next lane).  Offsets are formed as signed
    // numbers: a row origin before the tensor's start (padding) or a row outside the image wraps to an offset the
    // bounds check refuses, and reads zeros.  Columns outside the image are cleared on the way to LDS; the buffers are
    // reused from tile to tile, so every element is rewritten.
    static_assert(PITCH == 4 * 64, "a lane's 4 columns cover a staged row exactly");
    typedef uint2 stage_t[ROWS_W];
    uint32_t colmask[2];
#pragma unroll
    for (int d = 0; d < 2; ++d) {
        const int x = 4 * lane + 2 * d;
        colmask[d] = ((unsigned)(x - a.pad) < (unsigned)a.W ? 0x0000FFFFu : 0u) |
                     ((unsigned)(x + 1 - a.pad) < (unsigned)a.W ? 0xFFFF0000u : 0u);
    }
    auto tile_rows = [&](int tile, int& img, int& p0, int& row0) {
        uint32_t q, r;
        a.dX.divmod((uint32_t)tile, q, r);
        img = (int)q;
        p0 = (int)r * TN;
        row0 = (int)a.dOW.div((uint32_t)p0);
    };
    // Wave w stages the input rows w, w+4, ... of the tile, each in all C channels: stage slot i = k*C + c is input
    // row rr = w + 4k, channel c, staged row rr*C + c.  Returns the slots (bit i) fetched one element early.
    auto load_rows = [&](int tile, stage_t& st_reg) -> uint32_t {
        int img, p0, row0;
        tile_rows(tile < t_end ? tile : t_begin, img, p0, row0);
        const bool live = tile < t_end;
        const int iy_w = row0 * ST - a.pad + wave;
        const int origin_w = img * C * a.HW + iy_w * a.W - a.pad;  // element index of staged column 0, k = 0, c = 0
        uint32_t shifted = 0;
#pragma unroll
        for (int k = 0; k < RR_W; ++k) {
            const bool row_ok = live && wave + WAVES * k < IRMAX && (unsigned)(iy_w + WAVES * k) < (unsigned)a.H;
#pragma unroll
            for (int c = 0; c < C; ++c) {
                const int origin = origin_w + k * WAVES * a.W + c * a.HW;
                const int rowoff = row_ok ? (origin & ~1) * 2 : (int)kFarScalar;
                if (row_ok && (origin & 1)) shifted |= 1u << (k * C + c);
                // two dword loads, not one of 8 bytes: before the tensor's start (padding of the very first row) the bounds
                // check has to refuse one dword and pass the next
                // (a negative offset is replaced explicitly: left to wrap, it could be split into a register part and an
                // immediate part whose sum the bounds check forms in more than 32 bits)
                const int o0 = lane * 8 + rowoff, o1 = o0 + 4;
                st_reg[k * C + c].x = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(rin, o0 < 0 ? (int)kFarOffset : o0, 0, 0);
                st_reg[k * C + c].y = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(rin, o1 < 0 ? (int)kFarOffset : o1, 0, 0);
            }
        }
        return shifted;
    };
    auto store_rows = [&](int buf, const stage_t& st_reg, uint32_t shifted) {
        uint2* Bd = (uint2*)(Bs0 + buf * B_ELEMS) + wave * C * (PITCH / 4) + lane;
#pragma unroll
        for (int k = 0; k < RR_W; ++k) {
            if (wave + WAVES * k < IRMAX) {
#pragma unroll
                for (int c = 0; c < C; ++c) {
                    // shifted rows: staged dword = high half of its fetched dword, low half of the next one (lane 63's
                    // last column, 255, is never inside an image)
                    const int i = k * C + c;
                    const uint32_t sh = (shifted >> i) & 1u ? 16u : 0u;
                    const uint32_t nx = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)st_reg[i].x, 0x130 /* wave_shl:1 */, 0xf, 0xf, false);
                    const uint32_t lo = __builtin_amdgcn_alignbit(st_reg[i].y, st_reg[i].x, sh);
                    const uint32_t hi = __builtin_amdgcn_alignbit(nx, st_reg[i].y, sh);
                    Bd[(k * WAVES * C + c) * (PITCH / 4)] = make_uint2(lo & colmask[0], hi & colmask[1]);
                }
            }
        }
    };

    // each group's first tile is in flight while the filters are staged
    int tile = t_begin + grp;
    stage_t st_a;
    uint32_t sh_a = load_rows(tile, st_a);

    swin16_stage_filters<CFG>(As, bias_s, rfilt, a, m0, tid);
    // the extra row of both patch buffers stays zero
    if (tid < PITCH / 2) {
        ((uint32_t*)(Bs0 + SROWS * PITCH))[tid] = 0u;
        ((uint32_t*)(Bs0 + B_ELEMS + SROWS * PITCH))[tid] = 0u;
    }
    store_rows(grp, st_a, sh_a);
    __syncthreads();

    const __amdgpu_buffer_rsrc_t rout = make_rsrc(a.out, a.out_bytes);

    // lanes of the upper half whose line 2t+1 does not exist (odd number of lines) clear that operand
    const uint32_t last_pair_mask = (h && (NROW & 1)) ? 0u : 0xFFFFFFFFu;
    const int buf = grp;
    // Both groups make the same number of passes (the barriers are the workgroup's); a group without a tile idles.
    for (int first = t_begin; first < t_end; first += 2, tile += 2) {
        // rows of the group's next tile: they replace this tile's rows once the group is done with them
        const bool more = tile + 2 < t_end;
        if (more) sh_a = load_rows(tile + 2, st_a);

        if (tile < t_end) {
        int img, p0, row0;
        tile_rows(tile, img, p0, row0);
        const int p = p0 + wave * 32 + li;
        const bool p_ok = p < a.OHW;
        uint32_t oy, ox;
        a.dOW.divmod(p_ok ? (uint32_t)p : (uint32_t)p0, oy, ox);
        // the window's first element in line h: staged row (oy-row0)*ST*C + h, column ST*ox
        const elem_t* __restrict__ Bp = Bs0 + buf * B_ELEMS + (((int)oy - row0) * ST * C + h) * PITCH + ST * (int)ox;
        const elem_t* __restrict__ Ap = As + li * LDA + 8 * h;

        typename mma_t::acc_t acc[TMB][1];
#pragma unroll
        for (int mb = 0; mb < TMB; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mb][0][v] = 0.0f;

        const elem_t* const Bps[1] = {Bp};
        swin16_mma_loop<CFG>(Ap, Bps, last_pair_mask, acc);

        // activation: max(x, 0) (a NaN sum becomes 0, as in every other kernel) or the identity (a NaN stays a NaN)
        auto act = [&](float x) { return a.relu ? __builtin_fmaxf(x, 0.0f) : x; };
        if (a.out_nhwc) {
            // [N][OH][OW][K]: a lane's 4 consecutive channels of a pixel leave as one 8-byte store (K is a multiple of 4)
            const uint32_t vo = p_ok ? (uint32_t)((img * a.OHW + p) * a.K + m0 + 4 * h) * 2u : kFarOffset;
#pragma unroll
            for (int mb = 0; mb < TMB; ++mb)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4 bq = *(const float4*)&bias_s[mb * 32 + q * 8 + h * 4];
                    const float bv[4] = {bq.x, bq.y, bq.z, bq.w};
                    uint32_t pk[2];
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        const float x0 = act(acc[mb][0][4 * q + 2 * e] + bv[2 * e]);
                        const float x1 = act(acc[mb][0][4 * q + 2 * e + 1] + bv[2 * e + 1]);
                        pk[e] = (uint32_t)Prec<DT>::from_f32(x0) | ((uint32_t)Prec<DT>::from_f32(x1) << 16);
                    }
                    const int kr = mb * 32 + q * 8;
                    const uint32_t o = (m0 + kr + 4 * h < a.K) ? vo : kFarOffset;
                    __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2_t, make_uint2(pk[0], pk[1])), rout, (int)o, kr * 2, 0);
                }
        } else {
        // byte offset of (image, channel m0 + 4h, pixel); the rows of a lane follow in steps of 1 and 5 channels
        uint32_t vo = p_ok ? (uint32_t)(img * a.K * a.OHW + p + (m0 + 4 * h) * a.OHW) * 2u : kFarOffset;
        const uint32_t step1 = (uint32_t)a.OHW * 2u, step5 = 5u * step1;
        const bool full = m0 + TM <= a.K;
#pragma unroll
        for (int mb = 0; mb < TMB; ++mb)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 bq = *(const float4*)&bias_s[mb * 32 + q * 8 + h * 4];
                const float bv[4] = {bq.x, bq.y, bq.z, bq.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int kr = mb * 32 + q * 8 + e;  // row of the tile, without the lane half's 4
                    const float x = act(acc[mb][0][4 * q + e] + bv[e]);
                    const uint32_t o = (full || m0 + kr + 4 * h < a.K) ? vo : kFarOffset;
                    buffer_store_elem<elem_t>(Prec<DT>::from_f32(x), rout, o);
                    if (p_ok) vo += e == 3 ? step5 : step1;
                }
            }
        }
        }
        if (first + 2 >= t_end) break;  // no group has a further tile
        __syncthreads();
        if (more) store_rows(buf, st_a, sh_a);
        __syncthreads();
    }
}

template <class CFG>
constexpr size_t swin16_lds_bytes()
{
    return sizeof(uint16_t) * ((size_t)CFG::TM * CFG::LDA + 2 * (size_t)CFG::B_ELEMS) + sizeof(float) * CFG::TM;
}

template <class CFG>
hipError_t swin16_launch(const Variant&, ConvArgs& a, hipStream_t s)
{
    constexpr size_t lds = swin16_lds_bytes<CFG>();
    static_assert(lds <= 160 * 1024, "filters and two patch buffers fit the LDS of a CU");
    const hipError_t e = ensure_dynamic_lds((const void*)swin16_kernel<CFG>, lds);
    if (e != hipSuccess) return e;
    const int tiles_img = (a.OHW + CFG::TN - 1) / CFG::TN;
    a.nsplit = 1;
    a.dX = make_fastdiv((uint32_t)tiles_img);
    const long long tiles = (long long)a.N * tiles_img;
    const int ktiles = (a.K + CFG::TM - 1) / CFG::TM;
    int wgs = 256 / ktiles;  // one workgroup per CU: the filters and two patch buffers fill its LDS
    if (wgs < 1) wgs = 1;
    if (wgs > tiles) wgs = (int)tiles;
    dim3 grid((unsigned)wgs, (unsigned)ktiles, 1);
    hipLaunchKernelGGL(swin16_kernel<CFG>, grid, dim3(CFG::NT), lds, s, a);
    return hipGetLastError();
}

template <class CFG>
bool swin16_valid(const Variant&, const conv_desc& d, int OH, int OW)
{
    if (d.dtype != CFG::DT || d.C != CFG::C || d.R != CFG::R || d.S != CFG::S || d.stride != CFG::ST) return false;
    if (d.pad < 0 || d.pad >= CFG::R || d.pad >= CFG::S) return false;
    // every input row a tile touches has a staged row, a staged row holds every column a window reads, and a lane's
    // two dwords cover a staged row's image part
    const int rows = swin16_rows_spanned(OH, OW, CFG::TN);
    if ((rows - 1) * CFG::ST + CFG::R > CFG::IRMAX) return false;
    if (CFG::ST * (OW - 1) + 4 * CFG::SQ > CFG::PITCH) return false;
    if (d.W + d.pad > CFG::PITCH - 1) return false;
    const long long in_bytes = (long long)d.N * d.C * d.H * d.W * 2, out_bytes = (long long)d.N * d.K * OH * OW * 2;
    if (in_bytes > kUgemmMaxBytes || out_bytes > kUgemmMaxBytes) return false;  // scalar + vector offsets never wrap
    if ((long long)d.K * CFG::C * CFG::R * CFG::S * 2 > kUgemmMaxBytes) return false;
    if ((d.flags & CONV_FLAG_OUT_NHWC) && (d.K % 4) != 0) return false;  // 8-byte stores of 4 channels
    const long long tiles_img = ((long long)OH * OW + CFG::TN - 1) / CFG::TN;
    if ((long long)d.N * tiles_img > (1LL << 30)) return false;
    if ((d.K + CFG::TM - 1) / CFG::TM > 256) return false;
    // a channel tile mostly empty wastes the staged filters' space and the MFMA rows
    if (CFG::TM > 32 && (d.K % CFG::TM) != 0 && (d.K % CFG::TM) <= CFG::TM - 32) return false;
    return true;
}

template <class CFG>
void swin16_register(std::vector<Variant>& out)
{
    Variant v;
    char buf[160];
    snprintf(buf, sizeof buf, "swin_%s_%dx%ds%d_c%d_M%dN%d", dtype_name(CFG::DT), CFG::R, CFG::S, CFG::ST, CFG::C, CFG::TM,
             CFG::TN);
    v.name = buf;
    v.dtype = CFG::DT;
    v.split = 1;
    v.tm = CFG::TM;
    v.tn = CFG::TN;
    v.tk = CFG::KP;
    v.threads = CFG::NT;
    v.family = FAM_FIRSTLAYER;
    v.specificity = 6;
    v.traits = TRAIT_PLANAR_TO_NHWC;
    v.valid = &swin16_valid<CFG>;
    v.launch = &swin16_launch<CFG>;
    out.push_back(v);
}

}  // namespace convfwd
