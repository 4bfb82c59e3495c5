// Implicit-GEMM forward convolution on channel-innermost tensors, fp16 / bf16 storage.
//
// The paper's second graph-level optimisation is to insert explicit data-format conversions so that each operation
// sees the layout it runs best with (Section 3, "Graph-level Optimizations").  For the 16-bit MFMA the best layout is
// channel-innermost: a lane feeds 8 consecutive reduction elements per instruction, and with
//     in   [N][H][W][C]      (NHWC)
//     filt [K][R][S][C]      (KRSC)
//     reduction index q = (r*S + s)*C + c
// those 8 elements are 16 contiguous, 16-byte aligned bytes of both operands (C % 8 == 0).  So both tiles are staged
// with 16-byte loads and 16-byte LDS writes and nothing is transposed, packed or permuted on the way:
//   * filter tile: rows of the [K][Q] filter matrix, as in the other implicit-GEMM kernels;
//   * patch tile [pixel][k]: TK/8 consecutive lanes fetch the TK channels-at-one-tap of one pixel (one or two
//     contiguous runs); the pixel's window origin is a per-thread constant, the tap offset ((r*W + s)*C + c) is
//     recomputed per step from the lane's own reduction index (a handful of vector instructions, which 16-bit MFMAs
//     hide), zero padding is the per-pixel tap mask of the scalar-offset kernel.
// MFMA step, fragment double buffering across the barrier and the split/NCHW epilogue are shared with the other
// implicit-GEMM kernels; a channel-innermost output goes through an LDS transposition so that every pixel's TM
// output channels leave as contiguous 16-byte stores.
#pragma once

#include <type_traits>

#include "ugemm_kernel.h"

namespace convfwd {

template <class CFG>
constexpr size_t nhwc_lds_bytes()
{
    const size_t pipe = 2 * sizeof(uint16_t) * ((size_t)CFG::A_ELEMS + (size_t)CFG::B_ELEMS);
    const size_t epi = sizeof(uint16_t) * (size_t)CFG::TN * (CFG::TM + 8);
    return pipe > epi ? pipe : epi;
}

template <class CFG, int PADMODE>
__global__ __launch_bounds__(CFG::NT) void nhwc_kernel(ConvArgs a)
{
    typedef uint16_t elem_t;
    constexpr int DT = CFG::DT, MB = CFG::MB, WN = CFG::WN, BM = CFG::BM, BN = CFG::BN, TK = CFG::TK;
    constexpr int NT = CFG::NT, TM = CFG::TM, TN = CFG::TN, LDA = CFG::LDA, LDB = CFG::LDB, KPL = CFG::KPL;
    typedef Mma<DT, MB> mma_t;
    typedef typename mma_t::acc_t acc_t;
    constexpr int ACC_N = sizeof(acc_t) / sizeof(float);
    static_assert(DT != CONV_F32 && !CFG::B_KMAJOR && CFG::AVEC && MB == 32, "16-bit storage, 32x32 blocks, 16-byte loads");
    constexpr int KV = TK / 8;                 // 16-byte vectors per pixel row of the patch tile / per filter tile row
    constexpr int B_LOADS = TN * KV / NT;      // patch vectors per thread and step
    constexpr int B_PSTEP = NT / KV;           // tile pixels between two loads of one thread
    constexpr int A_LOADS = TM * KV / NT;
    constexpr int A_RSTEP = NT / KV;
    static_assert(NT % KV == 0 && (TN * KV) % NT == 0 && (TM * KV) % NT == 0, "whole loads per thread");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    elem_t* const As0 = (elem_t*)smem_raw;                    // [2][A_ELEMS]
    elem_t* const Bs0 = As0 + 2 * CFG::A_ELEMS;               // [2][B_ELEMS]

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int lrow = lane % MB, kg = lane / MB;
    const int p0 = blockIdx.x * TN, m0 = blockIdx.y * TM;

    // the input is addressed from pad*(W+1) pixels before its start, so that every window origin is a non-negative offset
    const uint32_t shift_bytes = (uint32_t)(a.pad * (a.W + 1)) * (uint32_t)a.C * 2u;
    const __amdgpu_buffer_rsrc_t rin = make_rsrc((const char*)a.in - shift_bytes, a.in_bytes + shift_bytes);
    const __amdgpu_buffer_rsrc_t rfilt = make_rsrc(a.filt, a.filt_bytes);

    const int total_steps = (a.Q + TK - 1) / TK;
    const int step_begin = blockIdx.z * a.steps_per_split;
    int step_end = step_begin + a.steps_per_split;
    if (step_end > total_steps) step_end = total_steps;

    // ---- per-thread constants ---------------------------------------------------------------------------------------
    const int koct = tid % KV;                 // which 8 reduction elements of a step's TK this thread moves
    const int row0 = tid / KV;                 // first tile pixel (patch) / first tile row (filter) of this thread
    uint32_t b_voff[B_LOADS], tapbad[B_LOADS];
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i) {
        const int p = p0 + row0 + i * B_PSTEP;
        const bool pvalid = p < a.P;
        uint32_t n_img, rem, oy, ox;
        a.dOHW.divmod(pvalid ? (uint32_t)p : 0u, n_img, rem);
        a.dOW.divmod(rem, oy, ox);
        const int iy0 = (int)oy * a.stride, ix0 = (int)ox * a.stride;
        b_voff[i] = pvalid ? (uint32_t)(((int)n_img * a.H + iy0) * a.W + ix0) * (uint32_t)a.C * 2u : kFarOffset;
        uint32_t bad = 0;
        if constexpr (PADMODE == PAD_TAPS) {
            for (int r = 0; r < a.R; ++r)
                for (int s = 0; s < a.S; ++s) {
                    const bool in_img = ((unsigned)(iy0 - a.pad + r) < (unsigned)a.H) && ((unsigned)(ix0 - a.pad + s) < (unsigned)a.W);
                    if (!in_img) bad |= 1u << (r * a.S + s);
                }
        } else if constexpr (PADMODE == PAD_ROWCOL) {
            for (int s = 0; s < a.S; ++s)
                if (!((unsigned)(ix0 - a.pad + s) < (unsigned)a.W)) bad |= 1u << s;
            for (int r = 0; r < a.R; ++r)
                if (!((unsigned)(iy0 - a.pad + r) < (unsigned)a.H)) bad |= 1u << (16 + r);
        }
        tapbad[i] = bad;
    }
    uint32_t a_voff[A_LOADS];
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) {
        const int row = row0 + i * A_RSTEP;
        a_voff[i] = (m0 + row < a.K) ? (uint32_t)((m0 + row) * a.Q + koct * 8) * 2u : kFarOffset;
    }
    const int a_lds0 = row0 * LDA + koct * 8;   // + i * A_RSTEP * LDA
    const int b_lds0 = row0 * LDB + koct * 8;   // + i * B_PSTEP * LDB

    // two register sets: the loads of step t+3 are issued while those of step t+2 are still in flight (an L2 round trip
    // under load outlasts one step of a 128x128x64 tile about four times; with one set in flight the step waits for it)
    uint4 a_vec[2][A_LOADS], b_vec[2][B_LOADS];

    auto load_tiles = [&](auto setc, int step) {
        constexpr int set = decltype(setc)::value;
        const int q = step * TK + koct * 8;     // this thread's reduction index in this step
        const bool k_ok = q < a.Q;              // vectors never straddle the end: Q is a multiple of 8
        const uint32_t a_soff = (uint32_t)(step * TK) * 2u;
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i) {
            const u32x4 t = __builtin_amdgcn_raw_buffer_load_b128(rfilt, (int)(k_ok ? a_voff[i] : kFarOffset), (int)a_soff, 0);
            a_vec[set][i] = make_uint4(t.x, t.y, t.z, t.w);
        }
        uint32_t tap, c, r, s;
        a.dC.divmod(k_ok ? (uint32_t)q : 0u, tap, c);
        a.dS.divmod(tap, r, s);
        const uint32_t koff = ((r * (uint32_t)a.W + s) * (uint32_t)a.C + c) * 2u;
#pragma unroll
        for (int i = 0; i < B_LOADS; ++i) {
            uint32_t far = k_ok ? 0u : 1u;
            if constexpr (PADMODE == PAD_TAPS) far |= (tapbad[i] >> tap) & 1u;
            if constexpr (PADMODE == PAD_ROWCOL) far |= ((tapbad[i] >> s) | (tapbad[i] >> (16u + r))) & 1u;
            const uint32_t vo = (far << 31) | (b_voff[i] + koff);
            const u32x4 t = __builtin_amdgcn_raw_buffer_load_b128(rin, (int)vo, 0, 0);
            b_vec[set][i] = make_uint4(t.x, t.y, t.z, t.w);
        }
    };

    auto store_tiles = [&](auto bufc) {  // register set and LDS buffer have the step's parity
        constexpr int buf = decltype(bufc)::value, set = buf;
        elem_t* As = As0 + buf * CFG::A_ELEMS;
        elem_t* Bs = Bs0 + buf * CFG::B_ELEMS;
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i) *(uint4*)&As[a_lds0 + i * A_RSTEP * LDA] = a_vec[set][i];
#pragma unroll
        for (int i = 0; i < B_LOADS; ++i) *(uint4*)&Bs[b_lds0 + i * B_PSTEP * LDB] = b_vec[set][i];
    };

    acc_t acc[BM][BN];
#pragma unroll
    for (int bm = 0; bm < BM; ++bm)
#pragma unroll
        for (int bn = 0; bn < BN; ++bn)
#pragma unroll
            for (int v = 0; v < ACC_N; ++v) acc[bm][bn][v] = 0.0f;

    const int fa_row0 = (wm * BM * MB + lrow) * LDA + kg * KPL;
    const int fb_col0 = wn * BN * MB + lrow;

    // same pipeline as the scalar-offset kernel: fragments of step t+1 are fetched behind the barrier while the last
    // MFMAs of step t, which need registers only, cover the LDS latency
    constexpr int NU = igemm_units<CFG>();
    constexpr int TAILU = NU >= 4 ? NU / 4 : 1;
    auto body = [&](auto bufc, int step, IgemmFrags<CFG>& fc, IgemmFrags<CFG>& fn) {
        constexpr int buf = decltype(bufc)::value;
        const bool more = step + 1 < step_end;
        igemm_mma_range<CFG, 0, NU - TAILU>(fc, acc);
        if (more) store_tiles(std::integral_constant<int, buf ^ 1>{});
        __syncthreads();
        if (more) igemm_read_frags<CFG>(As0 + (buf ^ 1) * CFG::A_ELEMS, Bs0 + (buf ^ 1) * CFG::B_ELEMS, fn, fa_row0, fb_col0, kg);
        // unconditional (a conditional load makes every later wait assume the worst): past the reduction's end the
        // loads are pointed out of range, past a split's end they fetch the next split's data, which is not used
        load_tiles(std::integral_constant<int, buf ^ 1>{}, step + 3);
        __builtin_amdgcn_sched_barrier(0);
        igemm_mma_range<CFG, NU - TAILU, NU>(fc, acc);
    };

    if (step_begin < step_end) {
        IgemmFrags<CFG> f0, f1;
        load_tiles(std::integral_constant<int, 0>{}, step_begin);
        store_tiles(std::integral_constant<int, 0>{});
        __syncthreads();
        igemm_read_frags<CFG>(As0, Bs0, f0, fa_row0, fb_col0, kg);
        load_tiles(std::integral_constant<int, 1>{}, step_begin + 1);
        load_tiles(std::integral_constant<int, 0>{}, step_begin + 2);
        for (int step = step_begin; step < step_end; step += 2) {
            body(std::integral_constant<int, 0>{}, step, f0, f1);
            if (step + 1 < step_end) body(std::integral_constant<int, 1>{}, step + 1, f1, f0);
        }
    }

    if (a.nsplit > 1 || !a.out_nhwc) {
        igemm_epilogue<CFG>(a, acc, p0, m0, wm, wn, lane, lrow);  // fp32 partial sums, or the [N][K][OH][OW] output
        return;
    }

    // ---- channel-innermost output: out[p][k] is a [P][K] matrix; transpose the tile through LDS ---------------------
    constexpr int LDC = TM + 8;
    elem_t* const Cs = (elem_t*)smem_raw;  // [TN][LDC]
    const __amdgpu_buffer_rsrc_t rbias = make_rsrc(a.bias, a.bias ? (uint32_t)a.K * 4u : 0u);
    float bias_r[BM][ACC_N];
#pragma unroll
    for (int bm = 0; bm < BM; ++bm)
#pragma unroll
        for (int v = 0; v < ACC_N; ++v)
            bias_r[bm][v] = buffer_load_elem<float>(rbias, (uint32_t)(m0 + wm * BM * MB + bm * MB + acc_row<MB>(v, lane)) * 4u);
    __syncthreads();  // every wave is done reading the operand tiles
#pragma unroll
    for (int bm = 0; bm < BM; ++bm)
#pragma unroll
        for (int bn = 0; bn < BN; ++bn) {
            const int pl = wn * BN * MB + bn * MB + lrow;
#pragma unroll
            for (int v4 = 0; v4 < ACC_N / 4; ++v4) {
                // accumulator registers 4*v4 .. 4*v4+3 of a lane are four consecutive output channels
                uint32_t h[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float x = acc[bm][bn][v4 * 4 + e] + bias_r[bm][v4 * 4 + e];
                    if (a.relu) x = x > 0.0f ? x : 0.0f;
                    h[e] = Prec<DT>::from_f32(x);
                }
                const int kl = wm * BM * MB + bm * MB + acc_row<MB>(v4 * 4, lane);
                *(uint2*)&Cs[pl * LDC + kl] = make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
            }
        }
    __syncthreads();
    const __amdgpu_buffer_rsrc_t rout = make_rsrc(a.out, a.out_bytes);
    constexpr int CV = TM / 8;  // 16-byte vectors per pixel
#pragma unroll
    for (int i = 0; i < TN * CV / NT; ++i) {
        const int v = i * NT + tid;
        const int pl = v / CV, kv = v % CV;
        const uint4 x = *(const uint4*)&Cs[pl * LDC + kv * 8];
        const int p = p0 + pl, k = m0 + kv * 8;
        const bool ok = p < a.P && k < a.K;  // K is a multiple of 8: a vector is in or out as a whole
        __builtin_amdgcn_raw_buffer_store_b128(u32x4{x.x, x.y, x.z, x.w}, rout,
                                               (int)(ok ? ((uint32_t)p * (uint32_t)a.K + (uint32_t)k) * 2u : kOutOfRange), 0, 0);
    }
}

// ---------------------------------------------------------------------------
// host side of a variant
// ---------------------------------------------------------------------------
template <class CFG, int PADMODE>
hipError_t nhwc_launch(const Variant& v, ConvArgs& a, hipStream_t s)
{
    constexpr size_t lds = nhwc_lds_bytes<CFG>();
    const hipError_t e = ensure_dynamic_lds((const void*)nhwc_kernel<CFG, PADMODE>, lds);
    if (e != hipSuccess) return e;
    const int total_steps = (a.Q + CFG::TK - 1) / CFG::TK;
    a.nsplit = v.split;
    a.steps_per_split = (total_steps + v.split - 1) / v.split;
    dim3 grid((unsigned)((a.P + CFG::TN - 1) / CFG::TN), (unsigned)((a.K + CFG::TM - 1) / CFG::TM), (unsigned)v.split);
    hipLaunchKernelGGL((nhwc_kernel<CFG, PADMODE>), grid, dim3(CFG::NT), lds, s, a);
    return hipGetLastError();
}

template <class CFG, int PADMODE>
bool nhwc_valid(const Variant& v, const conv_desc& d, int OH, int OW)
{
    if (d.dtype != CFG::DT) return false;
    if (!(d.flags & CONV_FLAG_IN_NHWC) || !(d.flags & CONV_FLAG_FILT_KRSC)) return false;
    if ((d.C % 8) != 0) return false;
    if ((d.flags & CONV_FLAG_OUT_NHWC) && (d.K % 8) != 0) return false;
    const long long Q = (long long)d.C * d.R * d.S, P = (long long)d.N * OH * OW;
    if (PADMODE == PAD_NONE && d.pad != 0) return false;
    if (PADMODE == PAD_TAPS && (d.pad == 0 || d.R * d.S > 32)) return false;
    if (PADMODE == PAD_ROWCOL && (d.pad == 0 || d.R * d.S <= 32 || d.R > 16 || d.S > 16)) return false;
    const long long in_bytes = ((long long)d.N * d.H * d.W + (long long)d.pad * (d.W + 1)) * d.C * 2;
    if (in_bytes > kUgemmMaxBytes || (long long)d.K * Q * 2 > kUgemmMaxBytes) return false;
    const int kcap = ((d.K + 31) / 32) * 32;
    if (CFG::TM > kcap) return false;
    if (CFG::TM == 96 && (d.K % 96) != 0) return false;
    const long long pcap = ((P + 63) / 64) * 64;
    if (CFG::TN > pcap && CFG::TM > 32) return false;  // the smallest channel tile stays valid however few the pixels
    const long long steps = (Q + CFG::TK - 1) / CFG::TK;
    if (v.split > 1 && steps < 2LL * v.split) return false;
    if (v.split > 1 && (long long)d.K * P * 4 >= (1LL << 32)) return false;
    if (d.K > 65535LL * CFG::TM) return false;
    return true;
}

template <class CFG, int PADMODE>
void nhwc_register_one(std::vector<Variant>& out, std::initializer_list<int> splits)
{
    for (int sk : splits) {
        Variant v;
        char buf[160];
        snprintf(buf, sizeof buf, "nhwc_%s_M%dN%dK%d_w%dx%d_%s", dtype_name(CFG::DT), CFG::TM, CFG::TN, CFG::TK, CFG::WM, CFG::WN,
                 PADMODE == PAD_NONE ? "p0" : PADMODE == PAD_TAPS ? "pt" : "prc");
        v.name = buf;
        if (sk > 1) v.name += "_sk" + std::to_string(sk);
        v.dtype = CFG::DT;
        v.split = sk;
        v.tm = CFG::TM;
        v.tn = CFG::TN;
        v.tk = CFG::TK;
        v.threads = CFG::NT;
        v.family = FAM_NHWC;
        v.specificity = 2;
        v.traits = TRAIT_REGISTER_OPERANDS;
        v.valid = &nhwc_valid<CFG, PADMODE>;
        v.launch = &nhwc_launch<CFG, PADMODE>;
        out.push_back(v);
    }
}

template <class CFG>
void nhwc_register(std::vector<Variant>& out, std::initializer_list<int> splits)
{
    nhwc_register_one<CFG, PAD_NONE>(out, splits);
    nhwc_register_one<CFG, PAD_TAPS>(out, splits);
    nhwc_register_one<CFG, PAD_ROWCOL>(out, splits);
}

}  // namespace convfwd
