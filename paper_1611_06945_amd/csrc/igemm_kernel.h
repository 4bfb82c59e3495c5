// Implicit-GEMM forward convolution on MFMA for gfx950.
//
// GEMM view of the layer the paper defines (Section 2 "Background"; Section 3
// "Metaprogramming for NN Convolutions" calls convolution a generalised
// matrix-matrix product):
//     Out[K x P] = Filt[K x Q] * Patch[Q x P]
//     P = N*OH*OW (pixels), Q = C*R*S (reduction), Patch[(c,r,s),(n,oy,ox)] =
//     in[n, c, oy*stride-pad+r, ox*stride-pad+s] or 0 outside the image.
// The Patch matrix is never materialised: each workgroup gathers its Q-step x
// pixel tile straight from the NCHW input into LDS, the filter tile (rows of the
// KCRS tensor are already rows of Filt) beside it, and feeds MFMA from LDS.  The
// activation and bias are applied on the accumulator as it is written out
// (Section 3 "Graph-level Optimizations": the fusion is always done).
//
// Tile parameters are template constants, the counterpart of the paper's tuning
// string (register blocking BM x BN MFMA blocks per wave, WM x WN waves per
// workgroup, reduction step TK, vector width = 16-byte loads where the shape
// allows).  Tile loaders are unrolled from the cooperative-load rule (ceil(W/N)
// loads, only the last one guarded).
#pragma once

#include "common.h"

namespace convfwd {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Buffer descriptors let the hardware do the bounds test of a guarded tile load: a load whose byte offset is not
// below `bytes` returns zero, so a lane that must not read (padding, ragged tile edge) is simply pointed out of
// range -- no branch and no exec-mask juggling around the load (the paper's point about keeping conditionals out
// of the unrolled load sequence, Section 3 "Metaprogramming for NN Convolutions").
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}
constexpr uint32_t kOutOfRange = 0xFFFFFFFFu;

template <typename E>
__device__ __forceinline__ E buffer_load_elem(__amdgpu_buffer_rsrc_t r, uint32_t byte_off)
{
    if constexpr (sizeof(E) == 4)
        return __builtin_bit_cast(E, __builtin_amdgcn_raw_buffer_load_b32(r, (int)byte_off, 0, 0));
    else
        return (E)__builtin_amdgcn_raw_buffer_load_b16(r, (int)byte_off, 0, 0);
}
// Stores through a descriptor: a store whose offset is out of range is dropped by the hardware.
template <typename E>
__device__ __forceinline__ void buffer_store_elem(E v, __amdgpu_buffer_rsrc_t r, uint32_t byte_off)
{
    if constexpr (sizeof(E) == 4)
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, v), r, (int)byte_off, 0, 0);
    else
        __builtin_amdgcn_raw_buffer_store_b16((uint16_t)v, r, (int)byte_off, 0, 0);
}
__device__ __forceinline__ uint4 buffer_load_vec(__amdgpu_buffer_rsrc_t r, uint32_t byte_off)
{
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_off, 0, 0);
    return make_uint4(v.x, v.y, v.z, v.w);
}

// ---------------------------------------------------------------------------
// storage types
// ---------------------------------------------------------------------------
template <int DT>
struct Prec;

template <>
struct Prec<CONV_F32> {
    typedef float elem_t;
    static constexpr int KPACK = 1;  // reduction elements one lane feeds to one MFMA
    static __device__ __forceinline__ elem_t from_f32(float x) { return x; }
    static __device__ __forceinline__ float to_f32(elem_t x) { return x; }
};

template <>
struct Prec<CONV_F16> {
    typedef uint16_t elem_t;  // raw IEEE binary16 patterns
    static constexpr int KPACK = 8;
    static __device__ __forceinline__ elem_t from_f32(float x)
    {
        _Float16 h = (_Float16)x;  // v_cvt_f16_f32, round to nearest even
        return __builtin_bit_cast(uint16_t, h);
    }
    static __device__ __forceinline__ float to_f32(elem_t x) { return (float)__builtin_bit_cast(_Float16, x); }
    // two values rounded and packed (a in the low half): one v_cvt_pk_f16_f32
    static __device__ __forceinline__ uint32_t pack2_from_f32(float a, float b)
    {
        typedef float f32x2_t __attribute__((ext_vector_type(2)));
        typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{a, b}, f16x2_t));
    }
};

template <>
struct Prec<CONV_BF16> {
    typedef uint16_t elem_t;  // raw bfloat16 patterns (upper half of a binary32)
    static constexpr int KPACK = 8;
    static __device__ __forceinline__ elem_t from_f32(float x)
    {
        __bf16 h = (__bf16)x;  // v_cvt_pk_bf16_f32 (gfx950): round to nearest even, a NaN stays a NaN
        return __builtin_bit_cast(uint16_t, h);
    }
    static __device__ __forceinline__ float to_f32(elem_t x) { return __builtin_bit_cast(float, (uint32_t)x << 16); }
    // two values rounded and packed (a in the low half): one v_cvt_pk_bf16_f32
    static __device__ __forceinline__ uint32_t pack2_from_f32(float a, float b)
    {
        typedef float f32x2_t __attribute__((ext_vector_type(2)));
        typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{a, b}, bf16x2_t));
    }
};

// ---------------------------------------------------------------------------
// MFMA wrappers.  MB is the block edge (32 -> 32x32 block, 16 -> 16x16 block).
// Lane l supplies row (l % MB) of the A block and column (l % MB) of the B block
// for reduction group (l / MB); the accumulator holds column (l % MB).
// ---------------------------------------------------------------------------
template <int DT, int MB>
struct Mma;

template <>
struct Mma<CONV_F32, 32> {
    typedef f32x16 acc_t;
    static __device__ __forceinline__ acc_t run(float a, float b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
    }
};
template <>
struct Mma<CONV_F32, 16> {
    typedef f32x4 acc_t;
    static __device__ __forceinline__ acc_t run(float a, float b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
};
template <>
struct Mma<CONV_F16, 32> {
    typedef f32x16 acc_t;
    static __device__ __forceinline__ acc_t run(uint4 a, uint4 b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0,
                                                      0, 0);
    }
};
template <>
struct Mma<CONV_F16, 16> {
    typedef f32x4 acc_t;
    static __device__ __forceinline__ acc_t run(uint4 a, uint4 b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0,
                                                      0, 0);
    }
};
template <>
struct Mma<CONV_BF16, 32> {
    typedef f32x16 acc_t;
    static __device__ __forceinline__ acc_t run(uint4 a, uint4 b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c,
                                                       0, 0, 0);
    }
};
template <>
struct Mma<CONV_BF16, 16> {
    typedef f32x4 acc_t;
    static __device__ __forceinline__ acc_t run(uint4 a, uint4 b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c,
                                                       0, 0, 0);
    }
};

// Row of the MB x MB block that accumulator register v of lane `lane` holds
// (the column is lane % MB).
template <int MB>
__device__ __forceinline__ int acc_row(int v, int lane)
{
    if constexpr (MB == 32)
        return (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
    else
        return (lane >> 4) * 4 + v;
}

// MODE_GATHER: any descriptor.  MODE_POINTWISE: R = S = 1, stride 1, no padding (the image is the GEMM operand as it is).
enum { MODE_GATHER = 0, MODE_POINTWISE = 1 };

// ---------------------------------------------------------------------------
// compile-time geometry of one variant
// ---------------------------------------------------------------------------
template <int DT_, int MB_, int WM_, int WN_, int BM_, int BN_, int TK_, bool AVEC_, int MODE_>
struct IgemmCfg {
    static constexpr int DT = DT_, MB = MB_, WM = WM_, WN = WN_, BM = BM_, BN = BN_, TK = TK_, MODE = MODE_;
    static constexpr bool AVEC = AVEC_;
    typedef typename Prec<DT>::elem_t elem_t;
    static constexpr int NT = 64 * WM * WN;                 // threads per workgroup
    static constexpr int TM = WM * BM * MB;                 // output channels per workgroup
    static constexpr int TN = WN * BN * MB;                 // pixels per workgroup
    static constexpr int VEC = 16 / (int)sizeof(elem_t);    // elements per 16-byte access
    static constexpr int KGRP = 64 / MB;                    // lane groups along the reduction
    static constexpr int KPL = TK / KGRP;                   // reduction elements per lane group per step
    static constexpr int KPACK = Prec<DT>::KPACK;
    static constexpr int NMMA = KPL / KPACK;                // MFMAs per block pair per step
    static constexpr bool B_KMAJOR = (DT == CONV_F32);      // LDS patch tile [k][pixel] (fp32) or [pixel][k] (16-bit)
    static constexpr int LDA = TK + VEC;                    // padded so 16-byte rows fall on distinct banks
    static constexpr int LDB = B_KMAJOR ? TN + 4 : TK + VEC;
    static constexpr int A_ELEMS = TM * LDA;
    static constexpr int B_ELEMS = B_KMAJOR ? TK * LDB : TN * LDB;
    // gather: each thread owns one pixel column and, per step, NCH chunks of CHW consecutive reduction indices
    static constexpr int GROUPS = NT / TN;
    static constexpr int CHW = B_KMAJOR ? TK / GROUPS : 8;
    static constexpr int NCH = (TK / CHW) / GROUPS;
    // cooperative-load plans of the tile loaders
    static constexpr CoopPlan planAv = coop_plan(NT, TM * TK / VEC);  // filter tile by 16-byte vectors
    static constexpr CoopPlan planAs = coop_plan(NT, TM * TK);        // filter tile by single elements
    static constexpr CoopPlan planBv = coop_plan(NT, TK * TN / 4);    // pointwise patch tile by 4-pixel vectors
    static_assert(NT % TN == 0, "a thread must keep one pixel column");
    static_assert(TK % KGRP == 0 && KPL % KPACK == 0 && NMMA >= 1, "reduction step does not fit the MFMA shape");
    static_assert(!B_KMAJOR || (KPL % 4 == 0), "fp32 path reads A four reduction elements at a time");
    static_assert(CHW >= 1 && NCH >= 1 && NCH * GROUPS * CHW == TK, "gather chunks must tile the reduction step");
    static_assert(TK % VEC == 0, "vector loads along the reduction");
    static_assert(MODE != MODE_POINTWISE || (B_KMAJOR && (NT % (TN / 4) == 0)), "pointwise mode: fp32, fixed pixel vector");
};

// One reduction step of a wave: its BM x BN accumulator blocks advance by the TK reduction elements held in the LDS
// tiles A ([row][k]) and B ([k][pixel] for fp32, [pixel][k] for 16-bit storage).  All operand fragments of the step are
// requested from LDS first, so the LDS latency overlaps the MFMA chain.
template <class CFG, class ACC>
__device__ __forceinline__ void igemm_compute(const typename CFG::elem_t* __restrict__ A, const typename CFG::elem_t* __restrict__ B,
                                              ACC (&acc)[CFG::BM][CFG::BN], int a_row0, int b_col0, int kg)
{
    constexpr int MB = CFG::MB, BM = CFG::BM, BN = CFG::BN, LDA = CFG::LDA, LDB = CFG::LDB, KPL = CFG::KPL, NMMA = CFG::NMMA;
    typedef Mma<CFG::DT, MB> mma_t;
    if constexpr (CFG::B_KMAJOR) {
        f32x4 af[KPL / 4][BM];
        float bf[KPL][BN];
#pragma unroll
        for (int ii = 0; ii < KPL / 4; ++ii)
#pragma unroll
            for (int bm = 0; bm < BM; ++bm) af[ii][bm] = *(const f32x4*)&A[a_row0 + bm * MB * LDA + ii * 4];
#pragma unroll
        for (int kk = 0; kk < KPL; ++kk)
#pragma unroll
            for (int bn = 0; bn < BN; ++bn) bf[kk][bn] = B[(kg * KPL + kk) * LDB + b_col0 + bn * MB];
#pragma unroll
        for (int kk = 0; kk < KPL; ++kk)
#pragma unroll
            for (int bm = 0; bm < BM; ++bm)
#pragma unroll
                for (int bn = 0; bn < BN; ++bn) acc[bm][bn] = mma_t::run(af[kk / 4][bm][kk % 4], bf[kk][bn], acc[bm][bn]);
    } else {
        uint4 af[NMMA][BM], bf[NMMA][BN];
#pragma unroll
        for (int i = 0; i < NMMA; ++i) {
#pragma unroll
            for (int bm = 0; bm < BM; ++bm) af[i][bm] = *(const uint4*)&A[a_row0 + bm * MB * LDA + i * 8];
#pragma unroll
            for (int bn = 0; bn < BN; ++bn) bf[i][bn] = *(const uint4*)&B[(b_col0 + bn * MB) * LDB + kg * KPL + i * 8];
        }
#pragma unroll
        for (int i = 0; i < NMMA; ++i)
#pragma unroll
            for (int bm = 0; bm < BM; ++bm)
#pragma unroll
                for (int bn = 0; bn < BN; ++bn) acc[bm][bn] = mma_t::run(af[i][bm], bf[i][bn], acc[bm][bn]);
    }
}

// The same step in two halves, for kernels that keep the operand fragments of the next step in registers while the
// matrix pipe still works on the current one: igemm_read_frags fetches every fragment of a step from LDS,
// igemm_mma_range<U0, U1> issues the MFMAs of reduction units [U0, U1) of the step (a unit is one reduction element
// per lane group for fp32, one 8-element packet for 16-bit storage; CFG-wide count: igemm_units<CFG>()).
template <class CFG, bool KMAJOR = CFG::B_KMAJOR>
struct IgemmFrags;
template <class CFG>
struct IgemmFrags<CFG, true> {
    f32x4 a[CFG::KPL / 4][CFG::BM];
    float b[CFG::KPL][CFG::BN];
};
template <class CFG>
struct IgemmFrags<CFG, false> {
    uint4 a[CFG::NMMA][CFG::BM], b[CFG::NMMA][CFG::BN];
};
template <class CFG>
constexpr int igemm_units()
{
    return CFG::B_KMAJOR ? CFG::KPL : CFG::NMMA;
}

template <class CFG>
__device__ __forceinline__ void igemm_read_frags(const typename CFG::elem_t* __restrict__ A, const typename CFG::elem_t* __restrict__ B,
                                                 IgemmFrags<CFG>& f, int a_row0, int b_col0, int kg)
{
    constexpr int MB = CFG::MB, BM = CFG::BM, BN = CFG::BN, LDA = CFG::LDA, LDB = CFG::LDB, KPL = CFG::KPL, NMMA = CFG::NMMA;
    if constexpr (CFG::B_KMAJOR) {
#pragma unroll
        for (int ii = 0; ii < KPL / 4; ++ii)
#pragma unroll
            for (int bm = 0; bm < BM; ++bm) f.a[ii][bm] = *(const f32x4*)&A[a_row0 + bm * MB * LDA + ii * 4];
#pragma unroll
        for (int kk = 0; kk < KPL; ++kk)
#pragma unroll
            for (int bn = 0; bn < BN; ++bn) f.b[kk][bn] = B[(kg * KPL + kk) * LDB + b_col0 + bn * MB];
    } else {
#pragma unroll
        for (int i = 0; i < NMMA; ++i) {
#pragma unroll
            for (int bm = 0; bm < BM; ++bm) f.a[i][bm] = *(const uint4*)&A[a_row0 + bm * MB * LDA + i * 8];
#pragma unroll
            for (int bn = 0; bn < BN; ++bn) f.b[i][bn] = *(const uint4*)&B[(b_col0 + bn * MB) * LDB + kg * KPL + i * 8];
        }
    }
}

template <class CFG, int U0, int U1, class ACC>
__device__ __forceinline__ void igemm_mma_range(const IgemmFrags<CFG>& f, ACC (&acc)[CFG::BM][CFG::BN])
{
    constexpr int BM = CFG::BM, BN = CFG::BN;
    typedef Mma<CFG::DT, CFG::MB> mma_t;
#pragma unroll
    for (int u = U0; u < U1; ++u)
#pragma unroll
        for (int bm = 0; bm < BM; ++bm)
#pragma unroll
            for (int bn = 0; bn < BN; ++bn) {
                if constexpr (CFG::B_KMAJOR)
                    acc[bm][bn] = mma_t::run(f.a[u / 4][bm][u % 4], f.b[u][bn], acc[bm][bn]);
                else
                    acc[bm][bn] = mma_t::run(f.a[u][bm], f.b[u][bn], acc[bm][bn]);
            }
}

// Epilogue shared by the implicit-GEMM kernels: the accumulator blocks of one wave go out either as fp32 partial sums
// of this reduction split ([split][K][P], finished by the fixed-order second pass) or, with bias and activation applied
// and rounded once to the storage type, as the NKHW output (paper, Section 3 "Graph-level Optimizations").
template <class CFG, class ACC>
__device__ __forceinline__ void igemm_epilogue(const ConvArgs& a, ACC (&acc)[CFG::BM][CFG::BN], int p0, int m0, int wm, int wn,
                                               int lane, int lrow)
{
    typedef typename CFG::elem_t elem_t;
    constexpr int DT = CFG::DT, MB = CFG::MB, BM = CFG::BM, BN = CFG::BN;
    constexpr int ACC_N = sizeof(ACC) / sizeof(float);
    constexpr uint32_t ES = sizeof(elem_t);
    // Pixel coordinates of this lane's accumulator columns.
    int e_p[BN];
    uint32_t e_img[BN], e_pix[BN];
#pragma unroll
    for (int bn = 0; bn < BN; ++bn) {
        e_p[bn] = p0 + wn * BN * MB + bn * MB + lrow;
        a.dOHW.divmod(e_p[bn] < a.P ? (uint32_t)e_p[bn] : 0u, e_img[bn], e_pix[bn]);
    }
    if (a.nsplit > 1) {
        // partial sums of this split, [split][K][P] fp32; the fixed-order second pass applies bias and activation
        const __amdgpu_buffer_rsrc_t rws = make_rsrc(a.ws + (size_t)blockIdx.z * a.K * a.P, (uint32_t)a.K * a.P * 4u);
#pragma unroll
        for (int bm = 0; bm < BM; ++bm)
#pragma unroll
            for (int v = 0; v < ACC_N; ++v) {
                const int k = m0 + wm * BM * MB + bm * MB + acc_row<MB>(v, lane);
#pragma unroll
                for (int bn = 0; bn < BN; ++bn) {
                    const bool ok = k < a.K && e_p[bn] < a.P;
                    buffer_store_elem<float>(acc[bm][bn][v], rws, ok ? (uint32_t)(k * a.P + e_p[bn]) * 4u : kOutOfRange);
                }
            }
    } else {
        // bias of every accumulator row of this lane is fetched up front (a null bias reads as zeros)
        const __amdgpu_buffer_rsrc_t rbias = make_rsrc(a.bias, a.bias ? (uint32_t)a.K * 4u : 0u);
        float bias_r[BM][ACC_N];
#pragma unroll
        for (int bm = 0; bm < BM; ++bm)
#pragma unroll
            for (int v = 0; v < ACC_N; ++v) {
                const int k = m0 + wm * BM * MB + bm * MB + acc_row<MB>(v, lane);
                bias_r[bm][v] = buffer_load_elem<float>(rbias, (uint32_t)k * 4u);
            }
        const __amdgpu_buffer_rsrc_t rout = make_rsrc(a.out, a.out_bytes);
#pragma unroll
        for (int bm = 0; bm < BM; ++bm)
#pragma unroll
            for (int v = 0; v < ACC_N; ++v) {
                const int k = m0 + wm * BM * MB + bm * MB + acc_row<MB>(v, lane);
#pragma unroll
                for (int bn = 0; bn < BN; ++bn) {
                    float x = acc[bm][bn][v] + bias_r[bm][v];
                    if (a.relu) x = x > 0.0f ? x : 0.0f;
                    const bool ok = k < a.K && e_p[bn] < a.P;
                    buffer_store_elem<elem_t>(Prec<DT>::from_f32(x), rout,
                                              ok ? (uint32_t)((e_img[bn] * a.K + k) * a.OHW + e_pix[bn]) * ES : kOutOfRange);
                }
            }
    }
}

template <class CFG>
__global__ __launch_bounds__(CFG::NT) void igemm_kernel(ConvArgs a)
{
    typedef typename CFG::elem_t elem_t;
    constexpr int DT = CFG::DT, MB = CFG::MB, WN = CFG::WN, BM = CFG::BM, BN = CFG::BN, TK = CFG::TK;
    constexpr int NT = CFG::NT, TM = CFG::TM, TN = CFG::TN, VEC = CFG::VEC, LDA = CFG::LDA, LDB = CFG::LDB;
    constexpr int KPL = CFG::KPL, NMMA = CFG::NMMA, CHW = CFG::CHW, NCH = CFG::NCH, GROUPS = CFG::GROUPS;
    typedef Mma<DT, MB> mma_t;
    typedef typename mma_t::acc_t acc_t;
    constexpr int ACC_N = sizeof(acc_t) / sizeof(float);

    __shared__ __attribute__((aligned(16))) elem_t As[2][CFG::A_ELEMS];
    __shared__ __attribute__((aligned(16))) elem_t Bs[2][CFG::B_ELEMS];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int lrow = lane % MB, kg = lane / MB;
    const int p0 = blockIdx.x * TN, m0 = blockIdx.y * TM;

    constexpr uint32_t ES = sizeof(elem_t);
    const __amdgpu_buffer_rsrc_t rin = make_rsrc(a.in, a.in_bytes);
    const __amdgpu_buffer_rsrc_t rfilt = make_rsrc(a.filt, a.filt_bytes);

    // reduction steps of this split
    const int total_steps = (a.Q + TK - 1) / TK;
    const int step_begin = blockIdx.z * a.steps_per_split;
    int step_end = step_begin + a.steps_per_split;
    if (step_end > total_steps) step_end = total_steps;

    // ---- per-thread constants of the patch gather -------------------------------------------
    // MODE_GATHER: one pixel column per thread.  MODE_POINTWISE: one 4-pixel vector per thread.
    int g_base = 0, g_iy0 = 0, g_ix0 = 0;
    bool g_pvalid = false;
    const int g_pl = (CFG::MODE != MODE_POINTWISE) ? (tid % TN) : (tid % (TN / 4)) * 4;
    const int g_grp = (CFG::MODE != MODE_POINTWISE) ? (tid / TN) : (tid / (TN / 4));
    {
        const int p = p0 + g_pl;
        g_pvalid = p < a.P;
        uint32_t n_img, rem, oy, ox;
        a.dOHW.divmod(g_pvalid ? (uint32_t)p : 0u, n_img, rem);
        if constexpr (CFG::MODE != MODE_POINTWISE) {
            a.dOW.divmod(rem, oy, ox);
            g_iy0 = (int)oy * a.stride - a.pad;
            g_ix0 = (int)ox * a.stride - a.pad;
            g_base = (int)n_img * a.C * a.HW + g_iy0 * a.W + g_ix0;
        } else {
            g_base = (int)n_img * a.C * a.HW + (int)rem;  // 1x1, stride 1, pad 0: pixel index == input index
        }
    }

    // ---- staging registers --------------------------------------------------------------------
    constexpr CoopPlan planAv = CFG::planAv, planAs = CFG::planAs, planBv = CFG::planBv;
    uint4 a_vec[CFG::AVEC ? planAv.loads : 1];
    elem_t a_sc[CFG::AVEC ? 1 : planAs.loads];
    elem_t b_reg[(CFG::MODE != MODE_POINTWISE) ? NCH : 1][(CFG::MODE != MODE_POINTWISE) ? CHW : 1];
    uint4 b_vec[(CFG::MODE == MODE_POINTWISE) ? planBv.loads : 1];

    auto load_tiles = [&](int step) {
        const int q0 = step * TK;
        // filter tile: rows m0.. of Filt, columns q0..q0+TK
        if constexpr (CFG::AVEC) {
#pragma unroll
            for (int i = 0; i < planAv.loads; ++i) {
                const int v = i * NT + tid;
                const bool in_tile = (i + 1 < planAv.loads || !planAv.last_guarded) ? true : (v < TM * TK / VEC);
                const int row = v / (TK / VEC), col = (v % (TK / VEC)) * VEC;
                const bool ok = in_tile && (m0 + row < a.K) && (q0 + col < a.Q);
                a_vec[i] = buffer_load_vec(rfilt, ok ? (uint32_t)((m0 + row) * a.Q + q0 + col) * ES : kOutOfRange);
            }
        } else {
#pragma unroll
            for (int i = 0; i < planAs.loads; ++i) {
                const int v = i * NT + tid;
                const bool in_tile = (i + 1 < planAs.loads || !planAs.last_guarded) ? true : (v < TM * TK);
                const int row = v / TK, col = v % TK;
                const bool ok = in_tile && (m0 + row < a.K) && (q0 + col < a.Q);
                a_sc[i] = buffer_load_elem<elem_t>(rfilt, ok ? (uint32_t)((m0 + row) * a.Q + q0 + col) * ES : kOutOfRange);
            }
        }
        // patch tile
        if constexpr (CFG::MODE == MODE_GATHER) {
#pragma unroll
            for (int j = 0; j < NCH; ++j) {
                const int q = q0 + (g_grp + j * GROUPS) * CHW;
                uint32_t c, rs, r, s;
                a.dRS.divmod((uint32_t)q, c, rs);
                a.dS.divmod(rs, r, s);
                int off = (int)c * a.HW + (int)r * a.W + (int)s;
                int ri = (int)r, si = (int)s;
#pragma unroll
                for (int e = 0; e < CHW; ++e) {
                    const bool ok = g_pvalid && (q + e < a.Q) && ((unsigned)(g_iy0 + ri) < (unsigned)a.H) &&
                                    ((unsigned)(g_ix0 + si) < (unsigned)a.W);
                    b_reg[j][e] = buffer_load_elem<elem_t>(rin, ok ? (uint32_t)(g_base + off) * ES : kOutOfRange);
                    ++si;
                    ++off;
                    if (si == a.S) {
                        si = 0;
                        off += a.W - a.S;
                        ++ri;
                        if (ri == a.R) {
                            ri = 0;
                            off += a.HW - a.R * a.W;
                        }
                    }
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < planBv.loads; ++i) {
                const int v = i * NT + tid;
                const bool in_tile = (i + 1 < planBv.loads || !planBv.last_guarded) ? true : (v < TK * TN / 4);
                const int krow = v / (TN / 4);
                const int c = q0 + krow;
                const bool ok = in_tile && g_pvalid && (c < a.C);
                b_vec[i] = buffer_load_vec(rin, ok ? (uint32_t)(g_base + c * a.HW) * ES : kOutOfRange);
            }
        }
    };

    auto store_tiles = [&](int buf) {
        if constexpr (CFG::AVEC) {
#pragma unroll
            for (int i = 0; i < planAv.loads; ++i) {
                const int v = i * NT + tid;
                const bool in_tile = (i + 1 < planAv.loads || !planAv.last_guarded) ? true : (v < TM * TK / VEC);
                const int row = v / (TK / VEC), col = (v % (TK / VEC)) * VEC;
                if (in_tile) *(uint4*)&As[buf][row * LDA + col] = a_vec[i];
            }
        } else {
#pragma unroll
            for (int i = 0; i < planAs.loads; ++i) {
                const int v = i * NT + tid;
                const bool in_tile = (i + 1 < planAs.loads || !planAs.last_guarded) ? true : (v < TM * TK);
                const int row = v / TK, col = v % TK;
                if (in_tile) As[buf][row * LDA + col] = a_sc[i];
            }
        }
        if constexpr (CFG::MODE != MODE_POINTWISE) {
#pragma unroll
            for (int j = 0; j < NCH; ++j) {
                const int kk = (g_grp + j * GROUPS) * CHW;
                if constexpr (CFG::B_KMAJOR) {
#pragma unroll
                    for (int e = 0; e < CHW; ++e) Bs[buf][(kk + e) * LDB + g_pl] = b_reg[j][e];
                } else {
                    uint4 pk;
                    pk.x = (uint32_t)b_reg[j][0] | ((uint32_t)b_reg[j][1] << 16);
                    pk.y = (uint32_t)b_reg[j][2] | ((uint32_t)b_reg[j][3] << 16);
                    pk.z = (uint32_t)b_reg[j][4] | ((uint32_t)b_reg[j][5] << 16);
                    pk.w = (uint32_t)b_reg[j][6] | ((uint32_t)b_reg[j][7] << 16);
                    *(uint4*)&Bs[buf][g_pl * LDB + kk] = pk;
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < planBv.loads; ++i) {
                const int v = i * NT + tid;
                const bool in_tile = (i + 1 < planBv.loads || !planBv.last_guarded) ? true : (v < TK * TN / 4);
                const int krow = v / (TN / 4);
                if (in_tile) *(uint4*)&Bs[buf][krow * LDB + g_pl] = b_vec[i];
            }
        }
    };

    acc_t acc[BM][BN];
#pragma unroll
    for (int bm = 0; bm < BM; ++bm)
#pragma unroll
        for (int bn = 0; bn < BN; ++bn)
#pragma unroll
            for (int v = 0; v < ACC_N; ++v) acc[bm][bn][v] = 0.0f;

    const int a_row0 = (wm * BM * MB + lrow) * LDA + kg * KPL;  // + bm*MB*LDA
    const int b_col0 = wn * BN * MB + lrow;                     // + bn*MB

    auto compute = [&](int buf) { igemm_compute<CFG>(As[buf], Bs[buf], acc, a_row0, b_col0, kg); };

    // ---- main loop: registers prefetch step t+1 while MFMA consumes step t from LDS ----------
    if (step_begin < step_end) {
        load_tiles(step_begin);
        store_tiles(0);
        __syncthreads();
        int buf = 0;
        for (int step = step_begin; step < step_end; ++step) {
            const bool more = step + 1 < step_end;
            if (more) load_tiles(step + 1);
            compute(buf);
            if (more) store_tiles(buf ^ 1);
            __syncthreads();
            buf ^= 1;
        }
    }

    igemm_epilogue<CFG>(a, acc, p0, m0, wm, wn, lane, lrow);
}

// ---------------------------------------------------------------------------
// host side of a variant
// ---------------------------------------------------------------------------
template <class CFG>
hipError_t igemm_launch(const Variant& v, ConvArgs& a, hipStream_t s)
{
    const int total_steps = (a.Q + CFG::TK - 1) / CFG::TK;
    a.nsplit = v.split;
    a.steps_per_split = (total_steps + v.split - 1) / v.split;
    dim3 grid((unsigned)((a.P + CFG::TN - 1) / CFG::TN), (unsigned)((a.K + CFG::TM - 1) / CFG::TM), (unsigned)v.split);
    hipLaunchKernelGGL(igemm_kernel<CFG>, grid, dim3(CFG::NT), 0, s, a);
    return hipGetLastError();
}

template <class CFG>
bool igemm_valid(const Variant& v, const conv_desc& d, int OH, int OW)
{
    if (d.dtype != CFG::DT) return false;
    const long long Q = (long long)d.C * d.R * d.S, P = (long long)d.N * OH * OW;
    if (CFG::AVEC && (Q % CFG::VEC) != 0) return false;
    if (CFG::MODE == MODE_POINTWISE) {
        if (d.R != 1 || d.S != 1 || d.stride != 1 || d.pad != 0 || ((d.H * d.W) % 4) != 0) return false;
    }
    // tiles much larger than the problem only waste MFMA work
    const int kcap = ((d.K + 31) / 32) * 32;
    if (CFG::TM > kcap && CFG::TM > 16) return false;
    if (CFG::TM == 96 && (d.K % 96) != 0) return false;
    const long long pcap = ((P + 63) / 64) * 64;
    if (CFG::TN > pcap) return false;
    // a split must leave every part at least two reduction steps
    const long long steps = (Q + CFG::TK - 1) / CFG::TK;
    if (v.split > 1 && steps < 2LL * v.split) return false;
    if (v.split > 1 && (long long)d.K * P * 4 >= (1LL << 32)) return false;  // one split's partial sums: 32-bit offsets
    if (d.K > 65535LL * CFG::TM) return false;
    return true;
}

template <class CFG>
void igemm_register(std::vector<Variant>& out, const char* family_tag, int family, int specificity,
                    std::initializer_list<int> splits)
{
    for (int sk : splits) {
        Variant v;
        char buf[160];
        snprintf(buf, sizeof buf, "%s_%s_M%dN%dK%d_w%dx%d_b%d%s", family_tag, dtype_name(CFG::DT), CFG::TM, CFG::TN,
                 CFG::TK, CFG::WM, CFG::WN, CFG::MB, CFG::AVEC ? "_v" : "_s");
        v.name = buf;
        if (sk > 1) v.name += "_sk" + std::to_string(sk);
        v.dtype = CFG::DT;
        v.split = sk;
        v.tm = CFG::TM;
        v.tn = CFG::TN;
        v.tk = CFG::TK;
        v.threads = CFG::NT;
        v.family = family;
        v.specificity = specificity + (CFG::AVEC ? 1 : 0);
        v.traits = CFG::AVEC ? 0u : TRAIT_SCALAR_LOADS;
        v.valid = &igemm_valid<CFG>;
        v.launch = &igemm_launch<CFG>;
        out.push_back(v);
    }
}

}  // namespace convfwd
