// Pointwise (1x1, stride 1, no padding) convolution on the plain formats for small and mid-sized operations: a GEMM
//     Out[K x P] = Filt[K x C] * X[C x P],   X[c][(n,pix)] = in[n][c][pix]
// whose whole operand set is a few megabytes, so that its run time is one round of memory latency plus the matrix
// work, provided every SIMD of the chip has a wave and every wave has all its loads in flight at once.
//   * Both operands go from global memory straight into MFMA registers -- no LDS staging, no barrier in the loop.  A lane
//     of a 32x32x2 MFMA feeds one filter value (row l % 32) and one input value (pixel l % 32) for channel l / 32 of
//     the step.  The reduction order is free, so lane half h takes channels 4h .. 4h+3 of a group of 8 over 4 MFMAs:
//     its four filter values are ONE 16-byte load of the [K][C] matrix, its four input values four 4-byte loads that
//     are contiguous along the pixels of the wave (128-byte runs of one channel plane).
//   * KW waves split the channels of one output tile (wave kw takes groups kw, kw + KW, ...): a 64 x 32 tile of the
//     benchmark's pointwise layer keeps 8 waves busy, and even an operation with 64 output tiles fills the chip with
//     KW = 16.  This replaces the reduction split over workgroups and its second launch.  Partial sums are added in
//     wave order through LDS (deterministic), then bias + activation + store.
//   * Loads run GD groups ahead through a ring of register slots; with few groups per wave everything is in flight
//     from the first instruction on.
//   * fp16 / bf16 storage: a lane of a 32x32x16 MFMA feeds 8 consecutive channels (8h .. 8h+7 of a group of 16).  Its
//     filter values are one 16-byte load; its input values lie one channel plane apart in [N][C][H][W], so they are
//     eight 2-byte loads (each contiguous along the pixels of the wave: 64-byte runs) put together in pairs.  That is
//     four times the load instructions of a layout with the channels innermost, which does not matter for the
//     operations this kernel is for: their run time is latency, not load issue.
#pragma once

#include "pwin_kernel.h"

namespace convfwd {

template <int DT_, int KW_, int TMB_, int NBW_, int GD_>
struct PwkCfg {
    static constexpr int DT = DT_, KW = KW_, TMB = TMB_, NBW = NBW_, GD = GD_;
    static constexpr int ES = DT == CONV_F32 ? 4 : 2;      // bytes per stored element
    static constexpr int GC = DT == CONV_F32 ? 8 : 16;     // channels per group (two lane halves x 4 or 8)
    static constexpr int HC = GC / 2;                      // channels of a lane half per group
    static constexpr int NT = 64 * KW;
    static_assert(NT <= 1024, "workgroup size");
    static constexpr int TM = 32 * TMB, TNP = 32 * NBW;
    static constexpr int RBP = TM + 4;  // floats per pixel in the reduction buffer (pixel pitch = 4 banks mod 64)
    static constexpr size_t LDS_BYTES = sizeof(float) * ((size_t)KW * TNP * RBP + TM);
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
};

// a.dX divides by the number of pixel tiles (set by the launcher)
template <class CFG>
__global__ __launch_bounds__(CFG::NT) void pwk_kernel(ConvArgs a)
{
    constexpr int DT = CFG::DT, KW = CFG::KW, TMB = CFG::TMB, NBW = CFG::NBW, GD = CFG::GD, NT = CFG::NT, TM = CFG::TM;
    constexpr int TNP = CFG::TNP, RBP = CFG::RBP, ES = CFG::ES, GC = CFG::GC, HC = CFG::HC;
    constexpr bool F32 = DT == CONV_F32;
    typedef typename Prec<DT>::elem_t elem_t;
    typedef Mma<DT, 32> mma_t;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int kw = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, h = lane >> 5;

    // ids b, b+8, ... run on one XCD: give each XCD a contiguous run of pixel tiles of (mostly) one channel tile
    const int PT = (int)a.dX.d, MT = (a.K + TM - 1) / TM, T = MT * PT;
    int logical;
    {
        const int b = blockIdx.x, x = b & 7, q = b >> 3;
        const int per = T >> 3, rem = T & 7;
        logical = x * per + (x < rem ? x : rem) + q;
    }
    uint32_t mt_u, pt_u;
    a.dX.divmod((uint32_t)logical, mt_u, pt_u);
    const int m0 = (int)mt_u * TM, p0 = (int)pt_u * TNP;

    const __amdgpu_buffer_rsrc_t rin = make_rsrc(a.in, a.in_bytes);
    const __amdgpu_buffer_rsrc_t rfilt = make_rsrc(a.filt, a.filt_bytes);

    // per-lane byte offsets at channel 0 of the lane's half (h selects channels HC*h .. HC*h + HC-1 of every group)
    uint32_t a_off[TMB], b_off[NBW];
#pragma unroll
    for (int mb = 0; mb < TMB; ++mb) {
        const int k = m0 + mb * 32 + li;
        a_off[mb] = k < a.K ? (uint32_t)(k * a.C + HC * h) * (uint32_t)ES : kOutOfRange;
    }
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb) {
        const int p = p0 + nb * 32 + li;
        uint32_t n, pix;
        a.dHW.divmod((uint32_t)(p < a.P ? p : 0), n, pix);
        b_off[nb] = p < a.P ? (uint32_t)(((int)n * a.C + HC * h) * a.HW + (int)pix) * (uint32_t)ES : kOutOfRange;
    }
    const int G = a.C / GC;                  // groups of GC channels
    const int NG = (G - kw + KW - 1) / KW;   // groups of this wave: kw, kw + KW, ...
    const uint32_t hw4 = (uint32_t)a.HW * (uint32_t)ES;  // bytes from one channel plane to the next

    u32x4 ar[GD][TMB];                       // fp32: 4 channels; 16-bit: 8 channels
    uint32_t br[GD][NBW][4];                 // fp32: 4 channels; 16-bit: 4 pairs of channels
    // loads of this wave's i-th group into ring slot `slot`; past the wave's last group every lane is pointed out of
    // range (the loads return zero and the products add nothing), so the sequence is the same for every wave
    auto load_group = [&](auto slot_c, int i) {
        constexpr int slot = decltype(slot_c)::value;
        const int g = kw + i * KW;
        const bool live = i < NG;
        const uint32_t ca = (uint32_t)g * 32u;              // GC channels along a filter row: 32 bytes in every type
        const uint32_t cb = (uint32_t)g * (uint32_t)GC * hw4;  // GC channel planes
#pragma unroll
        for (int mb = 0; mb < TMB; ++mb)
            ar[slot][mb] = __builtin_amdgcn_raw_buffer_load_b128(rfilt, (int)((live && a_off[mb] != kOutOfRange) ? a_off[mb] + ca : kOutOfRange), 0, 0);
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb) {
            const uint32_t base = (live && b_off[nb] != kOutOfRange) ? b_off[nb] + cb : kOutOfRange;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if constexpr (F32) {
                    br[slot][nb][j] = buffer_load_elem<uint32_t>(rin, base == kOutOfRange ? kOutOfRange : base + (uint32_t)j * hw4);
                } else {
                    const uint32_t lo = buffer_load_elem<uint16_t>(rin, base == kOutOfRange ? kOutOfRange : base + (uint32_t)(2 * j) * hw4);
                    const uint32_t hi = buffer_load_elem<uint16_t>(rin, base == kOutOfRange ? kOutOfRange : base + (uint32_t)(2 * j + 1) * hw4);
                    br[slot][nb][j] = lo | (hi << 16);
                }
            }
        }
    };

    typename mma_t::acc_t acc[TMB][NBW];
#pragma unroll
    for (int mb = 0; mb < TMB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mb][nb][v] = 0.0f;

    static_for<GD>([&](auto sc) { load_group(sc, decltype(sc)::value); });
    const int rounds = ((G + KW - 1) / KW + GD - 1) / GD;  // the same for every wave of the workgroup
    for (int r = 0; r < rounds; ++r) {
        static_for<GD>([&](auto sc) {
            constexpr int slot = decltype(sc)::value;
            if constexpr (F32) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int mb = 0; mb < TMB; ++mb)
#pragma unroll
                        for (int nb = 0; nb < NBW; ++nb) {
                            // (copies first: a bit cast applied directly to a vector element reads the vector's first element)
                            const uint32_t av = ar[slot][mb][j], bv = br[slot][nb][j];
                            acc[mb][nb] = mma_t::run(__builtin_bit_cast(float, av), __builtin_bit_cast(float, bv), acc[mb][nb]);
                        }
            } else {
#pragma unroll
                for (int mb = 0; mb < TMB; ++mb)
#pragma unroll
                    for (int nb = 0; nb < NBW; ++nb)
                        acc[mb][nb] = mma_t::run(make_uint4(ar[slot][mb].x, ar[slot][mb].y, ar[slot][mb].z, ar[slot][mb].w),
                                                 make_uint4(br[slot][nb][0], br[slot][nb][1], br[slot][nb][2], br[slot][nb][3]), acc[mb][nb]);
            }
            load_group(sc, (r + 1) * GD + slot);
        });
    }

    // ---- add the KW waves' partial sums in wave order, then bias + activation + store -------------------------------
    float* const red = (float*)smem_raw;  // [KW][TNP][RBP] + [TM] bias
#pragma unroll
    for (int mb = 0; mb < TMB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb) {
            float* dst = &red[(kw * TNP + nb * 32 + li) * RBP + mb * 32 + 4 * h];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const typename mma_t::acc_t& c = acc[mb][nb];
                *(f32x4*)&dst[8 * i] = f32x4{c[4 * i], c[4 * i + 1], c[4 * i + 2], c[4 * i + 3]};
            }
        }
    const __amdgpu_buffer_rsrc_t rbias = make_rsrc(a.bias, a.bias ? (uint32_t)a.K * 4u : 0u);
    const __amdgpu_buffer_rsrc_t rout = make_rsrc(a.out, a.out_bytes);
    if (tid < TM) red[KW * TNP * RBP + tid] = buffer_load_elem<float>(rbias, m0 + tid < a.K ? (uint32_t)(m0 + tid) * 4u : kOutOfRange);
    __syncthreads();
    // a thread keeps one pixel and walks down the channels four at a time; consecutive threads hold consecutive pixels
    constexpr int RG = TM / 4, CPT = NT / TNP;
    static_assert(CPT >= 1, "at least one thread per pixel of the tile");
    const float* bsm = &red[KW * TNP * RBP];
    const int col = tid % TNP, rg0 = tid / TNP;
    const int p = p0 + col;
    const bool pok = rg0 < CPT && p < a.P;
    uint32_t n, pix;
    a.dHW.divmod((uint32_t)(pok ? p : 0), n, pix);
    uint32_t o = (uint32_t)(((int)n * a.K + m0 + rg0 * 4) * a.HW + (int)pix) * (uint32_t)ES;
    const float* src = &red[col * RBP];
    for (int rg = rg0; rg < RG; rg += CPT) {
        f32x4 x = *(const f32x4*)&src[rg * 4];
#pragma unroll
        for (int q = 1; q < KW; ++q) x += *(const f32x4*)&src[q * TNP * RBP + rg * 4];
        const f32x4 bv = *(const f32x4*)&bsm[rg * 4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float y = x[i] + bv[i];
            if (a.relu) y = y > 0.0f ? y : 0.0f;
            const bool oki = pok && m0 + rg * 4 + i < a.K;
            buffer_store_elem<elem_t>(Prec<DT>::from_f32(y), rout, oki ? o + (uint32_t)i * hw4 : kOutOfRange);
        }
        o += 4u * CPT * hw4;
    }
}

template <class CFG>
hipError_t pwk_launch(const Variant&, ConvArgs& a, hipStream_t s)
{
    const hipError_t e = ensure_dynamic_lds((const void*)pwk_kernel<CFG>, CFG::LDS_BYTES);
    if (e != hipSuccess) return e;
    const int PT = (a.P + CFG::TNP - 1) / CFG::TNP, MT = (a.K + CFG::TM - 1) / CFG::TM;
    a.dX = make_fastdiv((uint32_t)PT);
    hipLaunchKernelGGL(pwk_kernel<CFG>, dim3((unsigned)(PT * MT)), dim3(CFG::NT), CFG::LDS_BYTES, s, a);
    return hipGetLastError();
}

template <class CFG>
bool pwk_valid(const Variant&, const conv_desc& d, int OH, int OW)
{
    if (d.dtype != CFG::DT || d.R != 1 || d.S != 1 || d.stride != 1 || d.pad != 0) return false;
    if (d.flags & ~(uint32_t)CONV_FLAG_RELU) return false;  // plain formats, no fused pool
    if ((d.C % CFG::GC) != 0) return false;
    const long long P = (long long)d.N * OH * OW;
    const long long tiles = ((P + CFG::TNP - 1) / CFG::TNP) * ((d.K + CFG::TM - 1) / CFG::TM);
    if (tiles > 0x7fffffffLL) return false;
    const long long lim = 1LL << 31;  // byte offsets are formed in 32 bits, with room for the look-ahead past the end
    if ((long long)d.N * d.C * d.H * d.W * 4 >= lim || (long long)d.K * d.C * 4 >= lim || (long long)d.K * P * 4 >= lim) return false;
    // a wave needs at least one group of channels
    if (d.C / CFG::GC < CFG::KW) return false;
    return true;
}

template <class CFG>
void pwk_register(std::vector<Variant>& out)
{
    Variant v;
    char buf[160];
    snprintf(buf, sizeof buf, "pwk_%s_M%dN%d_w%d_g%d", dtype_name(CFG::DT), CFG::TM, CFG::TNP, CFG::KW, CFG::GD);
    v.name = buf;
    v.dtype = CFG::DT;
    v.split = 1;
    v.tm = CFG::TM;
    v.tn = CFG::TNP;
    v.tk = CFG::GC * CFG::KW;
    v.threads = CFG::NT;
    v.family = FAM_POINTWISE;
    v.specificity = 6;
    v.traits = TRAIT_REGISTER_OPERANDS | TRAIT_WAVE_SPLIT;
    v.valid = &pwk_valid<CFG>;
    v.launch = &pwk_launch<CFG>;
    out.push_back(v);
}

}  // namespace convfwd
