// First-layer convolution with the 3x3 stride-2 max-pool that follows it computed in the same kernel (paper, Section 3
// "Graph-level Optimizations": an operation that only consumes the convolution's output is folded into it), fp16 / bf16
// storage.  The activation tensor of a first layer is the largest of the network and exists only to be pooled; here it
// never reaches memory.
//
// A workgroup owns a PTH x PTW tile of POOLED outputs of one image, i.e. a (2*PTH+1) x (2*PTW+1) tile of convolution
// outputs: the rows and columns shared by neighbouring tiles are computed by both (1.11x the multiply-adds for 9 x 9)
// instead of being handed over through memory.
//   * The input rows and columns the tile touches are staged once in LDS, [input row][channel][column], zero where the
//     padding or the image's end is; the filters are re-laid into [TM][KP] exactly as in the kernel without the pool
//     (swin16_kernel.h, whose filter staging and multiply loop are used here).
//   * Every wave multiplies NBW blocks of 32 convolution pixels of the tile for all TM channels (pixels are numbered
//     row-major inside the tile; the window origin is a per-lane LDS address, so the block's shape does not matter).
//     With 3 blocks x 3 channel blocks per wave a step reads 6 operand fragments for 9 MFMAs and the loop is bound by
//     the matrix units; with 1 block per wave (more waves) it is bound by LDS reads but hides latencies better, and is
//     the faster of the two.
//   * Bias, activation and rounding are applied to the convolution values, which then go to LDS as storage elements
//     [pixel][channel] (over the input rows, which are no longer needed); a second pass takes the 3x3 maxima, 8 channels
//     per thread, and writes the pooled tile, channel-innermost (16-byte stores) or channel-planar.  Rounding is
//     monotone, so the maximum of the rounded values is the rounded maximum: the result equals convolution, then pool.
//     Behind the activation every value is +0 or positive (a NaN sum has become 0), and the bit patterns of such fp16 /
//     bf16 values order like 16-bit integers: the maxima are taken two at a time with packed integer instructions.
#pragma once

#include "swin16_kernel.h"

// Compile-time experiment hook (0 in the product): bit 16 = workgroups write phase time stamps (100 MHz ticks) into the
// workspace, 8 per workgroup, when one is passed.
#ifndef SWINP_EXP
#define SWINP_EXP 0
#endif
#if SWINP_EXP & 16
#define SWINP_STAMP(i) do { if (tid == 0 && a.ws) ((unsigned long long*)a.ws)[(size_t)blockIdx.x * 8 + (i)] = wall_clock64(); } while (0)
#else
#define SWINP_STAMP(i) do { } while (0)
#endif

namespace convfwd {

template <int DT_, int C_, int R_, int S_, int ST_, int TMB_, int NBW_, int PTH_, int PTW_, int PITCH_>
struct SwinP16Cfg {
    static_assert(DT_ == CONV_F16 || DT_ == CONV_BF16, "16-bit storage only");
    static_assert(ST_ == 2 || ST_ == 4, "operand groups must stay dword aligned");
    static constexpr int DT = DT_, C = C_, R = R_, S = S_, ST = ST_, TMB = TMB_, NBW = NBW_, PTH = PTH_, PTW = PTW_, PITCH = PITCH_;
    static constexpr int CTH = 2 * PTH + 1, CTW = 2 * PTW + 1;  // convolution outputs under the pooled tile
    static constexpr int NPIX = CTH * CTW;
    static constexpr int NBLK = (NPIX + 31) / 32;    // 32-pixel blocks
    static constexpr int WAVES = (NBLK + NBW - 1) / NBW;
    static constexpr int NT = 64 * WAVES;
    static_assert(NT <= 1024 && NT % 128 == 0, "workgroup size (whole pairs of waves: the filter staging works on 128 threads)");
    static constexpr int TM = 32 * TMB;
    static constexpr int SQ = (S + 3) / 4;
    static constexpr int NROW = C * R;
    static constexpr int NPAIR = (NROW + 1) / 2;
    static constexpr int KSTEPS = (NPAIR * SQ + 1) / 2;
    static constexpr int KP = KSTEPS * 16;
    static constexpr int LDA = KP + 8;
    static constexpr int IR = (CTH - 1) * ST + R;          // input rows under the tile
    static constexpr int ICOLS = (CTW - 1) * ST + 4 * SQ;  // input columns a window of the tile can read
    static_assert(PITCH % 4 == 0 && PITCH >= ICOLS && PITCH <= 124, "32 lanes x 4 columns stage a row; lane 31 is never stored");
    static constexpr int SROWS = C * IR;
    // staging: a lane half takes one channel of one input row per pass; halves beyond a multiple of C stay idle, so
    // that a half keeps its channel and moves down RPP input rows from pass to pass
    static constexpr int UNITS = (2 * WAVES / C) * C;
    static_assert(UNITS > 0, "at least one input row (all channels) per pass");
    static constexpr int RPP = UNITS / C;                  // input rows per pass of the workgroup
    static constexpr int NIT = (IR + RPP - 1) / RPP;
    static constexpr int B_ELEMS = (SROWS + 1) * PITCH;    // one extra row: the lower line of a pair past the last line
    static constexpr int CPT = TM + 8;                     // channel pitch of the convolution tile in LDS
    static constexpr int T_ELEMS = NPIX * CPT;
    static constexpr int U_ELEMS = ((B_ELEMS > T_ELEMS ? B_ELEMS : T_ELEMS) + 7) / 8 * 8;  // the biases behind it stay 16-byte aligned
    static constexpr size_t LDS_BYTES = sizeof(uint16_t) * ((size_t)TM * LDA + U_ELEMS) + sizeof(float) * TM;
    static_assert(LDS_BYTES <= 160 * 1024, "filters, input rows / convolution tile and biases fit the LDS of a CU");
};

// a.dX divides by the tiles of one image, a.dY by the tile columns (set by the launcher)
template <class CFG>
__global__ __launch_bounds__(CFG::NT) void swinp16_kernel(ConvArgs a)
{
    typedef uint16_t elem_t;
    constexpr int DT = CFG::DT, C = CFG::C, ST = CFG::ST, TMB = CFG::TMB, NBW = CFG::NBW, PITCH = CFG::PITCH, PTH = CFG::PTH;
    constexpr int PTW = CFG::PTW, CTW = CFG::CTW, NPIX = CFG::NPIX, NT = CFG::NT, TM = CFG::TM, NROW = CFG::NROW, IR = CFG::IR;
    constexpr int LDA = CFG::LDA, SROWS = CFG::SROWS, NIT = CFG::NIT, UNITS = CFG::UNITS, RPP = CFG::RPP, CPT = CFG::CPT;
    typedef Mma<DT, 32> mma_t;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    elem_t* const As = (elem_t*)smem_raw;                 // [TM][LDA]
    elem_t* const Bs = As + TM * LDA;                     // [SROWS + 1][PITCH], later the convolution tile [NPIX][CPT]
    float* const bias_s = (float*)(Bs + CFG::U_ELEMS);    // [TM]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, h = lane >> 5;
    const int m0 = blockIdx.y * TM;
    SWINP_STAMP(0);

    // Workgroups are dealt to the 8 XCDs in turn: workgroup -> tile such that an XCD gets one contiguous run of tiles
    // (neighbouring tiles share input rows, and each XCD has its own L2).
    const int tiles_img = (int)a.dX.d;
    int tile;
    {
        const int T = a.N * tiles_img, b = (int)blockIdx.x, x = b & 7, q = b >> 3;
        const int per = T >> 3, rem = T & 7;
        tile = x * per + (x < rem ? x : rem) + q;
    }
    uint32_t img_u, t_u, ty_u, tx_u;
    a.dX.divmod((uint32_t)tile, img_u, t_u);
    a.dY.divmod(t_u, ty_u, tx_u);
    const int img = (int)img_u;
    const int py0 = (int)ty_u * PTH, px0 = (int)tx_u * PTW;      // first pooled output of the tile
    const int iy0 = 2 * py0 * ST - a.pad, ix0 = 2 * px0 * ST - a.pad;  // input element under staged row 0, column 0

    // whole dwords: the tensors' last elements may be the low halves of aligned dwords
    const __amdgpu_buffer_rsrc_t rin = make_rsrc(a.in, (a.in_bytes + 3u) & ~3u);
    const __amdgpu_buffer_rsrc_t rfilt = make_rsrc(a.filt, (a.filt_bytes + 3u) & ~3u);

    // ---- input rows of the tile -> registers ----------------------------------------------------------------------
    // Staged row sr = rr*C + c holds input row iy0 + rr of channel c; staged column x holds input column ix0 + x.  Lane
    // half u = 2*wave + h (the first UNITS of them) takes channel u % C of input rows u / C, + RPP, + 2*RPP, ...; a lane
    // takes 4 columns (8 bytes) of its row.  A row starts at any 2-byte alignment in memory, and a misaligned load runs
    // at a fraction of the rate: the two dwords are fetched from the aligned address at or one element before the row's
    // origin, and in the second case shifted by one element on the way to LDS (the missing half comes from the next
    // lane).  Offsets are formed as signed numbers: an origin before the tensor's start gives negative offsets, which
    // are replaced by one the bounds check refuses (reads zeros); rows outside the image get such an offset as well.
    // Columns outside the image are cleared on the way to LDS.
    uint32_t colmask[2];
#pragma unroll
    for (int d = 0; d < 2; ++d) {
        const int x = ix0 + 4 * li + 2 * d;
        colmask[d] = ((unsigned)x < (unsigned)a.W ? 0x0000FFFFu : 0u) | ((unsigned)(x + 1) < (unsigned)a.W ? 0xFFFF0000u : 0u);
    }
    const int unit = 2 * wave + h;
    const int u_rr = unit / C, u_c = unit - u_rr * C;
    const bool u_on = unit < UNITS;
    const int origin0 = (img * C + u_c) * a.HW + (iy0 + u_rr) * a.W + ix0;  // element under the unit's first row, column 0
    const int ostep = RPP * a.W;
    uint2 st_reg[NIT];
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int rr = u_rr + it * RPP;
        const bool row_ok = u_on && rr < IR && (unsigned)(iy0 + rr) < (unsigned)a.H;
        const int origin = origin0 + it * ostep;
        // two dword loads, not one of 8 bytes: before the tensor's start one dword has to read zero and the next has
        // to pass.  A negative offset is replaced explicitly: left to wrap, it could be split into a register part and
        // an immediate part whose sum the bounds check forms in more than 32 bits.
        const int o0 = row_ok ? li * 8 + (origin & ~1) * 2 : -1, o1 = row_ok ? o0 + 4 : -1;
        st_reg[it].x = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(rin, o0 < 0 ? (int)kFarOffset : o0, 0, 0);
        st_reg[it].y = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(rin, o1 < 0 ? (int)kFarOffset : o1, 0, 0);
    }

    SWINP_STAMP(1);
    swin16_stage_filters<CFG>(As, bias_s, rfilt, a, m0, tid);
    SWINP_STAMP(2);

    // ---- registers -> LDS -----------------------------------------------------------------------------------------
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int rr = u_rr + it * RPP;
        // shifted rows (odd origin): staged dword = high half of its fetched dword, low half of the next one.  The lane
        // after lane 31 belongs to the other row, and lane 31's columns (124..127) are past the staged row: never stored.
        const uint32_t sh = ((origin0 + it * ostep) & 1) ? 16u : 0u;
        const uint32_t nx = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)st_reg[it].x, 0x130 /* wave_shl:1 */, 0xf, 0xf, false);
        const uint32_t lo = __builtin_amdgcn_alignbit(st_reg[it].y, st_reg[it].x, sh);
        const uint32_t hi = __builtin_amdgcn_alignbit(nx, st_reg[it].y, sh);
        if (u_on && rr < IR && 4 * li < PITCH)
            *(uint2*)&Bs[(rr * C + u_c) * PITCH + 4 * li] = make_uint2(lo & colmask[0], hi & colmask[1]);
    }
    // the extra row: read (and masked) by the lanes whose lower line does not exist
    if (tid < PITCH / 2) ((uint32_t*)(Bs + SROWS * PITCH))[tid] = 0u;
    __syncthreads();
    SWINP_STAMP(3);

    // ---- this wave's NBW blocks of 32 convolution pixels ----------------------------------------------------------
    // pixel q of the tile, row-major; past the tile: computed (on pixel 0's window), not kept
    const elem_t* Bp[NBW];
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb) {
        const int q = (wave * NBW + nb) * 32 + li;
        const int qc = q < NPIX ? q : 0;
        const int ty = qc / CTW, tx = qc - ty * CTW;
        Bp[nb] = Bs + (ty * ST * C + h) * PITCH + ST * tx;
    }
    const elem_t* __restrict__ Ap = As + li * LDA + 8 * h;
    // lanes of the upper half whose line 2t+1 does not exist (odd number of lines) clear that operand
    const uint32_t last_pair_mask = (h && (NROW & 1)) ? 0u : 0xFFFFFFFFu;

    typename mma_t::acc_t acc[TMB][NBW];
#pragma unroll
    for (int mb = 0; mb < TMB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mb][nb][v] = 0.0f;
    swin16_mma_loop<CFG>(Ap, Bp, last_pair_mask, acc);

    // ---- bias, activation, rounding -> convolution tile in LDS (over the input rows) -----------------------------------
    SWINP_STAMP(4);
    __syncthreads();
    SWINP_STAMP(5);
    // activation: max(x, 0) (a NaN sum becomes 0, as in every other kernel) or the identity (a NaN stays a NaN)
    auto to_tile = [&](auto relu_c) {
        constexpr bool RELU = decltype(relu_c)::value;
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb) {
            const int q = (wave * NBW + nb) * 32 + li;
            if (q < NPIX) {
#pragma unroll
                for (int mb = 0; mb < TMB; ++mb)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const float4 bq = *(const float4*)&bias_s[mb * 32 + g * 8 + h * 4];
                        const float bv[4] = {bq.x, bq.y, bq.z, bq.w};
                        float x[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            x[e] = acc[mb][nb][4 * g + e] + bv[e];
                            if constexpr (RELU) x[e] = __builtin_fmaxf(x[e], 0.0f);
                        }
                        *(uint2*)&Bs[q * CPT + mb * 32 + g * 8 + h * 4] =
                            make_uint2(Prec<DT>::pack2_from_f32(x[0], x[1]), Prec<DT>::pack2_from_f32(x[2], x[3]));
                    }
            }
        }
    };
    if (a.relu) to_tile(std::true_type{}); else to_tile(std::false_type{});
    __syncthreads();
    SWINP_STAMP(6);

    // ---- 3x3 stride-2 maxima: a thread takes 8 channels of a pooled output ------------------------------------------------
    const __amdgpu_buffer_rsrc_t rout = make_rsrc(a.out, a.out_bytes);
    constexpr int CG = TM / 8, TASKS = PTH * PTW * CG;
    typedef short s16x2_t __attribute__((ext_vector_type(2)));
    const int npool = a.POH * a.POW;
    for (int e = tid; e < TASKS; e += NT) {
        const int pp = e / CG, cg = e - pp * CG;
        const int ly = pp / PTW, lx = pp - ly * PTW;
        const int py = py0 + ly, px = px0 + lx;
        const elem_t* const win = Bs + (2 * ly * CTW + 2 * lx) * CPT + cg * 8;
        uint32_t pk[4];
        if (a.relu) {
            // every value is +0 or positive and no NaN is left: their bit patterns order like signed 16-bit integers
            s16x2_t mi[4] = {s16x2_t{0, 0}, s16x2_t{0, 0}, s16x2_t{0, 0}, s16x2_t{0, 0}};
#pragma unroll
            for (int dy = 0; dy < 3; ++dy)
#pragma unroll
                for (int dx = 0; dx < 3; ++dx) {
                    const uint4 w = *(const uint4*)&win[(dy * CTW + dx) * CPT];
                    const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
                    for (int j = 0; j < 4; ++j) mi[j] = __builtin_elementwise_max(mi[j], __builtin_bit_cast(s16x2_t, ww[j]));
                }
#pragma unroll
            for (int j = 0; j < 4; ++j) pk[j] = __builtin_bit_cast(uint32_t, mi[j]);
        } else {
            float m[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) m[j] = -__builtin_inff();
#pragma unroll
            for (int dy = 0; dy < 3; ++dy)
#pragma unroll
                for (int dx = 0; dx < 3; ++dx) {
                    const uint4 w = *(const uint4*)&win[(dy * CTW + dx) * CPT];
                    const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const float x = Prec<DT>::to_f32((elem_t)(ww[j >> 1] >> (16 * (j & 1))));
                        m[j] = (x > m[j] || x != x) ? x : m[j];  // a NaN is the result
                    }
                }
#pragma unroll
            for (int j = 0; j < 4; ++j)
                pk[j] = (uint32_t)Prec<DT>::from_f32(m[2 * j]) | ((uint32_t)Prec<DT>::from_f32(m[2 * j + 1]) << 16);
        }
        const int k = m0 + cg * 8;
        const bool ok = py < a.POH && px < a.POW;
        if (a.out_nhwc) {
            // K is a multiple of 8: the 8 channels exist together
            const uint32_t o = ok && k < a.K ? (uint32_t)((img * npool + py * a.POW + px) * a.K + k) * 2u : kOutOfRange;
            __builtin_amdgcn_raw_buffer_store_b128(u32x4{pk[0], pk[1], pk[2], pk[3]}, rout, (int)o, 0, 0);
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t o = ok && k + j < a.K ? (uint32_t)((img * a.K + k + j) * npool + py * a.POW + px) * 2u : kOutOfRange;
                buffer_store_elem<elem_t>((elem_t)(pk[j >> 1] >> (16 * (j & 1))), rout, o);
            }
        }
    }
    SWINP_STAMP(7);
}

template <class CFG>
hipError_t swinp16_launch(const Variant&, ConvArgs& a, hipStream_t s)
{
    const hipError_t e = ensure_dynamic_lds((const void*)swinp16_kernel<CFG>, CFG::LDS_BYTES);
    if (e != hipSuccess) return e;
    const int TY = (a.POH + CFG::PTH - 1) / CFG::PTH, TX = (a.POW + CFG::PTW - 1) / CFG::PTW;
    a.nsplit = 1;
    a.dX = make_fastdiv((uint32_t)(TY * TX));
    a.dY = make_fastdiv((uint32_t)TX);
    const int ktiles = (a.K + CFG::TM - 1) / CFG::TM;
    dim3 grid((unsigned)(a.N * TY * TX), (unsigned)ktiles, 1);
    hipLaunchKernelGGL(swinp16_kernel<CFG>, grid, dim3(CFG::NT), CFG::LDS_BYTES, s, a);
    return hipGetLastError();
}

template <class CFG>
bool swinp16_valid(const Variant&, const conv_desc& d, int OH, int OW)
{
    if (!(d.flags & CONV_FLAG_MAXPOOL_3X3S2)) return false;  // this kernel writes the pooled tensor and nothing else
    if (d.dtype != CFG::DT || d.C != CFG::C || d.R != CFG::R || d.S != CFG::S || d.stride != CFG::ST) return false;
    if (d.pad < 0 || d.pad >= CFG::R || d.pad >= CFG::S) return false;
    if (OH < 3 || OW < 3) return false;
    const long long in_bytes = (long long)d.N * d.C * d.H * d.W * 2, out_bytes = (long long)d.N * d.K * OH * OW * 2;
    if (in_bytes > kUgemmMaxBytes || out_bytes > kUgemmMaxBytes) return false;  // signed byte offsets never wrap
    if ((long long)d.K * CFG::C * CFG::R * CFG::S * 2 > kUgemmMaxBytes) return false;
    if ((d.flags & CONV_FLAG_OUT_NHWC) && (d.K % 8) != 0) return false;  // 16-byte stores of 8 channels
    const int POH = (OH - 3) / 2 + 1, POW = (OW - 3) / 2 + 1;
    const long long tiles = (long long)d.N * ((POH + CFG::PTH - 1) / CFG::PTH) * ((POW + CFG::PTW - 1) / CFG::PTW);
    if (tiles > (1LL << 30)) return false;
    if ((d.K + CFG::TM - 1) / CFG::TM > 256) return false;
    // a channel tile mostly empty wastes the staged filters' space and the MFMA rows
    if (CFG::TM > 32 && (d.K % CFG::TM) != 0 && (d.K % CFG::TM) <= CFG::TM - 32) return false;
    return true;
}

template <class CFG>
void swinp16_register(std::vector<Variant>& out)
{
    Variant v;
    char buf[160];
    snprintf(buf, sizeof buf, "swinp_%s_%dx%ds%d_c%d_M%d_p%dx%d_w%d", dtype_name(CFG::DT), CFG::R, CFG::S, CFG::ST, CFG::C,
             CFG::TM, CFG::PTH, CFG::PTW, CFG::WAVES);
    v.name = buf;
    v.dtype = CFG::DT;
    v.split = 1;
    v.tm = CFG::TM;
    v.tn = CFG::NPIX;
    v.tk = CFG::KP;
    v.threads = CFG::NT;
    v.family = FAM_FIRSTLAYER;
    v.specificity = 7;
    v.traits = TRAIT_PLANAR_TO_NHWC | TRAIT_POOL_EPILOGUE;
    v.valid = &swinp16_valid<CFG>;
    v.launch = &swinp16_launch<CFG>;
    out.push_back(v);
}

}  // namespace convfwd
