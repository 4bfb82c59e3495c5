// Implicit-GEMM forward convolution whose tile loaders spend (almost) no vector-ALU instructions.
//
// Same GEMM view, tiles, LDS layouts, MFMA step and epilogue as igemm_kernel.h.  What differs is how the addresses of
// the filter tile and of the gathered patch tile are formed.  On this device an fp32 MFMA and a vector-ALU instruction
// of the same SIMD do not run side by side -- every vector instruction of any resident wave delays the matrix work by
// its own issue time -- so the index arithmetic of an im2col-style gather (the chain of constant multiplies, divides
// and modulos the paper describes in Section 3, "ND-Arrays") is moved off the vector unit entirely:
//   * a thread keeps one pixel column for the whole kernel; the byte offset of that pixel's window origin is computed
//     once and stays in a vector register;
//   * which reduction indices (c, r, s) a thread fetches in a step is the same for all 64 lanes of its wave, so their
//     offset c*H*W + r*W + s is computed on the scalar unit and handed to the load as its scalar offset;
//   * zero padding is one precomputed bit mask per thread (bit r*S+s set when tap (r,s) of this pixel falls outside
//     the image); a masked tap gets the top bit of its vector offset set, which the buffer bounds test turns into a
//     zero -- two vector instructions per element, none when the layer has no padding;
//   * LDS addresses are a per-thread base plus compile-time immediates (the double buffer is unrolled by two).
#pragma once

#include <type_traits>

#include "igemm_kernel.h"

namespace convfwd {

// how the zero padding is tested: PAD_NONE (pad == 0), PAD_TAPS (one mask bit per window tap, R*S <= 32),
// PAD_ROWCOL (one bit per window row and one per window column, R <= 16 and S <= 16)
enum { PAD_NONE = 0, PAD_TAPS = 1, PAD_ROWCOL = 2 };

constexpr uint32_t kFarOffset = 0x80000000u;   // vector offset of a lane that must read zero
constexpr uint32_t kFarScalar = 0x40000000u;   // scalar offset of a reduction index past the end
constexpr long long kUgemmMaxBytes = 0x3ff00000LL;  // tensors stay below 1 GiB so that the sums above never wrap

template <class CFG, int PADMODE, bool SV = false>
__global__ __launch_bounds__(CFG::NT) void ugemm_kernel(ConvArgs a)
{
    typedef typename CFG::elem_t elem_t;
    constexpr int DT = CFG::DT, MB = CFG::MB, WN = CFG::WN, BM = CFG::BM, BN = CFG::BN, TK = CFG::TK;
    constexpr int NT = CFG::NT, TM = CFG::TM, TN = CFG::TN, VEC = CFG::VEC, LDA = CFG::LDA, LDB = CFG::LDB;
    constexpr int KPL = CFG::KPL, CHW = CFG::CHW, NCH = CFG::NCH, GROUPS = CFG::GROUPS;
    typedef Mma<DT, MB> mma_t;
    typedef typename mma_t::acc_t acc_t;
    constexpr int ACC_N = sizeof(acc_t) / sizeof(float);
    constexpr uint32_t ES = sizeof(elem_t);
    static_assert(TN % 64 == 0, "the reduction indices a thread gathers must be the same for its whole wave");
    static_assert(NT % TK == 0 && NT % (TK / VEC) == 0, "filter tile rows advance by a constant per load");
    static_assert(!SV || (CFG::B_KMAJOR && CFG::AVEC && PADMODE == PAD_NONE && (CHW % 4) == 0 && NCH * CHW <= 32),
                  "s-vector gather: fp32, 16-byte filter loads, no padding");

    __shared__ __attribute__((aligned(16))) elem_t As[2][CFG::A_ELEMS];
    __shared__ __attribute__((aligned(16))) elem_t Bs[2][CFG::B_ELEMS];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int lrow = lane % MB, kg = lane / MB;
    const int p0 = blockIdx.x * TN, m0 = blockIdx.y * TM;

    // the input is addressed from pad*(W+1) elements before its start: the window origin of every pixel is then a
    // non-negative offset; the elements before the tensor belong to padding taps only, which are never fetched
    const uint32_t shift_bytes = (uint32_t)(a.pad * (a.W + 1)) * ES;
    const __amdgpu_buffer_rsrc_t rin = make_rsrc((const char*)a.in - shift_bytes, a.in_bytes + shift_bytes);
    const __amdgpu_buffer_rsrc_t rfilt = make_rsrc(a.filt, a.filt_bytes);

    const int Qeff = SV ? a.QP : a.Q;  // length of the reduction axis as this kernel lays it out
    const int total_steps = (Qeff + TK - 1) / TK;
    const int step_begin = blockIdx.z * a.steps_per_split;
    int step_end = step_begin + a.steps_per_split;
    if (step_end > total_steps) step_end = total_steps;

    // ---- per-thread constants of the patch gather ---------------------------------------------------------------
    const int g_pl = tid % TN;                                       // pixel column of the tile
    const int u_grp = __builtin_amdgcn_readfirstlane(tid / TN);      // which reduction chunks of a step: wave-uniform
    uint32_t b_voff;        // byte offset of the window origin, or kFarOffset for a pixel column past the end
    uint32_t tapbad = 0;    // PAD_TAPS: bit r*S+s; PAD_ROWCOL: bit s (columns) and bit 16+r (rows)
    {
        const int p = p0 + g_pl;
        const bool pvalid = p < a.P;
        uint32_t n_img, rem, oy, ox;
        a.dOHW.divmod(pvalid ? (uint32_t)p : 0u, n_img, rem);
        a.dOW.divmod(rem, oy, ox);
        const int iy0 = (int)oy * a.stride, ix0 = (int)ox * a.stride;  // window origin in the shifted addressing
        b_voff = pvalid ? (uint32_t)((int)n_img * a.C * a.HW + iy0 * a.W + ix0) * ES : kFarOffset;
        if constexpr (PADMODE == PAD_TAPS) {
            for (int r = 0; r < a.R; ++r)
                for (int s = 0; s < a.S; ++s) {
                    const bool in_img = ((unsigned)(iy0 - a.pad + r) < (unsigned)a.H) && ((unsigned)(ix0 - a.pad + s) < (unsigned)a.W);
                    if (!in_img) tapbad |= 1u << (r * a.S + s);
                }
        } else if constexpr (PADMODE == PAD_ROWCOL) {
            for (int s = 0; s < a.S; ++s)
                if (!((unsigned)(ix0 - a.pad + s) < (unsigned)a.W)) tapbad |= 1u << s;
            for (int r = 0; r < a.R; ++r)
                if (!((unsigned)(iy0 - a.pad + r) < (unsigned)a.H)) tapbad |= 1u << (16 + r);
        }
    }

    // ---- per-thread constants of the filter tile ------------------------------------------------------------------
    constexpr CoopPlan planAv = CFG::planAv, planAs = CFG::planAs;
    constexpr int A_LOADS = CFG::AVEC ? planAv.loads : planAs.loads;
    constexpr int A_W = CFG::AVEC ? VEC : 1;                 // elements per filter load
    constexpr int A_CPR = TK / A_W;                          // loads per tile row
    constexpr int A_ROWSTEP = NT / A_CPR;                    // tile rows between two loads of one thread
    const int a_row0 = tid / A_CPR, a_col = (tid % A_CPR) * A_W;
    uint32_t a_voff[A_LOADS];  // byte offset of (row, a_col) in the filter matrix, or kFarOffset
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) {
        const int row = a_row0 + i * A_ROWSTEP;
        const bool ok = row < TM && m0 + row < a.K;
        a_voff[i] = ok ? (uint32_t)((m0 + row) * a.Q + a_col) * ES : kFarOffset;
    }
    const int a_lds0 = a_row0 * LDA + a_col;                                   // + i * A_ROWSTEP * LDA
    const int b_lds0 = CFG::B_KMAJOR ? u_grp * CHW * LDB + g_pl               // + (j*GROUPS*CHW + e) * LDB
                                     : g_pl * LDB + u_grp * CHW;              // + j*GROUPS*CHW

    // s-vector layout: this thread's filter column q' = q0 + a_col as (c, r, s') of the padded axis, advanced step by step
    int sv_c = 0, sv_r = 0, sv_s = 0;
    int sv_left = 4;           // of the filter vectors in flight: how many leading columns are window columns
    uint32_t sv_keep = ~0u;    // of the patch elements in flight (uniform): bit j*CHW+e set when the column is a window column
    if constexpr (SV) {
        uint32_t c, rem, r, sp;
        a.dRSP.divmod((uint32_t)(step_begin * TK + a_col), c, rem);
        a.dSP.divmod(rem, r, sp);
        sv_c = (int)c; sv_r = (int)r; sv_s = (int)sp;
    }

    uint4 a_vec[CFG::AVEC ? A_LOADS : 1];
    elem_t a_sc[CFG::AVEC ? 1 : A_LOADS];
    elem_t b_reg[NCH][CHW];

    auto load_tiles = [&](int step) {
        const int q0 = step * TK;  // uniform
        const uint32_t a_soff = SV ? 0u : (uint32_t)q0 * ES;
        if constexpr (SV) {
            // columns (c, r, s'..s'+3) of the padded axis are filter elements (c, r, s'..s'+3) where s' + e < S, else zero
            const bool col_ok = sv_c < a.C;
            const uint32_t foff = (uint32_t)(sv_c * a.RS + sv_r * a.S + sv_s - a_col) * ES;  // a_voff already holds a_col
            sv_left = a.S - sv_s;  // window columns the vector really holds; the rest is cleared when it goes to LDS
#pragma unroll
            for (int i = 0; i < A_LOADS; ++i) {
                const uint32_t vo = col_ok ? a_voff[i] + foff : kFarOffset;
                const u32x4 t = __builtin_amdgcn_raw_buffer_load_b128(rfilt, (int)vo, 0, 0);
                a_vec[i] = make_uint4(t.x, t.y, t.z, t.w);
            }
            // advance by one step (TK columns) for the next call; steps are visited in order
            sv_s += TK;
            const int SP = 4 * a.SP4;
            while (sv_s >= SP) {
                sv_s -= SP;
                if (++sv_r == a.R) {
                    sv_r = 0;
                    ++sv_c;
                }
            }
        } else if (q0 + TK <= a.Q) {
            // whole step inside the reduction axis: no per-lane test at all
#pragma unroll
            for (int i = 0; i < A_LOADS; ++i) {
                if constexpr (CFG::AVEC) {
                    const u32x4 t = __builtin_amdgcn_raw_buffer_load_b128(rfilt, (int)a_voff[i], (int)a_soff, 0);
                    a_vec[i] = make_uint4(t.x, t.y, t.z, t.w);
                } else if constexpr (sizeof(elem_t) == 4) {
                    a_sc[i] = __builtin_bit_cast(elem_t, __builtin_amdgcn_raw_buffer_load_b32(rfilt, (int)a_voff[i], (int)a_soff, 0));
                } else {
                    a_sc[i] = (elem_t)__builtin_amdgcn_raw_buffer_load_b16(rfilt, (int)a_voff[i], (int)a_soff, 0);
                }
            }
        } else {
            // last, partial step: columns past the end of the filter row read as zero
            const bool col_ok = q0 + a_col < a.Q;
#pragma unroll
            for (int i = 0; i < A_LOADS; ++i) {
                const uint32_t vo = col_ok ? a_voff[i] : kFarOffset;
                if constexpr (CFG::AVEC) {
                    u32x4 t = __builtin_amdgcn_raw_buffer_load_b128(rfilt, (int)vo, (int)a_soff, 0);
                    if constexpr (sizeof(elem_t) == 4) {
                        // a row length that is no multiple of the vector: the vector's tail belongs to the next row
                        const int left = a.Q - (q0 + a_col);
                        if (left < 2) t.y = 0u;
                        if (left < 3) t.z = 0u;
                        if (left < 4) t.w = 0u;
                    }
                    a_vec[i] = make_uint4(t.x, t.y, t.z, t.w);
                } else if constexpr (sizeof(elem_t) == 4) {
                    a_sc[i] = __builtin_bit_cast(elem_t, __builtin_amdgcn_raw_buffer_load_b32(rfilt, (int)vo, (int)a_soff, 0));
                } else {
                    a_sc[i] = (elem_t)__builtin_amdgcn_raw_buffer_load_b16(rfilt, (int)vo, (int)a_soff, 0);
                }
            }
        }
        // patch tile: the reduction indices are uniform, so (c, r, s) and the offset live on the scalar unit
        if constexpr (SV) {
            uint32_t keep = 0u;
#pragma unroll
            for (int j = 0; j < NCH; ++j) {
                const int q = q0 + (u_grp + j * GROUPS) * CHW;  // a multiple of 4 in the padded axis
                uint32_t c, rem, r, sv;
                a.dRSP4.divmod((uint32_t)q >> 2, c, rem);
                a.dSP4.divmod(rem, r, sv);
                int ci = (int)c, ri = (int)r, svi = (int)sv;
#pragma unroll
                for (int v4 = 0; v4 < CHW / 4; ++v4) {
                    const int s0 = svi * 4;
                    const uint32_t soff = ci < a.C ? (uint32_t)(ci * a.HW + ri * a.W + s0) * ES : kFarScalar;
                    // four window columns at once; columns past the window are real neighbours (or read as zero past the
                    // end of the tensor) and are cleared when the tile goes to LDS -- not here, which would wait for the load
                    const u32x4 t = __builtin_amdgcn_raw_buffer_load_b128(rin, (int)b_voff, (int)soff, 0);
                    const uint32_t w4[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        b_reg[j][v4 * 4 + e] = __builtin_bit_cast(elem_t, w4[e]);
                        if (s0 + e < a.S) keep |= 1u << (j * CHW + v4 * 4 + e);
                    }
                    if (++svi == a.SP4) {
                        svi = 0;
                        if (++ri == a.R) {
                            ri = 0;
                            ++ci;
                        }
                    }
                }
            }
            sv_keep = keep;
        } else
#pragma unroll
        for (int j = 0; j < NCH; ++j) {
            const int q = q0 + (u_grp + j * GROUPS) * CHW;
            uint32_t c, rs, r, s;
            a.dRS.divmod((uint32_t)q, c, rs);
            a.dS.divmod(rs, r, s);
            int off = (int)c * a.HW + (int)r * a.W + (int)s;
            int ri = (int)r, si = (int)s;
#pragma unroll
            for (int e = 0; e < CHW; ++e) {
                const uint32_t soff = (q + e < a.Q) ? (uint32_t)off * ES : kFarScalar;
                uint32_t vo = b_voff;
                if constexpr (PADMODE == PAD_TAPS) {
                    const uint32_t bad = __builtin_amdgcn_ubfe(tapbad, (uint32_t)(ri * a.S + si), 1u);
                    vo = (bad << 31) | b_voff;
                } else if constexpr (PADMODE == PAD_ROWCOL) {
                    const uint32_t sel = (1u << si) | (1u << (16 + ri));  // uniform
                    vo = (tapbad & sel) ? kFarOffset : b_voff;
                }
                if constexpr (sizeof(elem_t) == 4)
                    b_reg[j][e] = __builtin_bit_cast(elem_t, __builtin_amdgcn_raw_buffer_load_b32(rin, (int)vo, (int)soff, 0));
                else
                    b_reg[j][e] = (elem_t)__builtin_amdgcn_raw_buffer_load_b16(rin, (int)vo, (int)soff, 0);
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
    };

    auto store_tiles = [&](auto bufc) {
        constexpr int buf = decltype(bufc)::value;
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i) {
            const bool in_tile = (a_row0 + i * A_ROWSTEP) < TM;  // false only for the last load of a ragged plan
            if constexpr (CFG::AVEC) {
                if constexpr (SV) {
                    if (sv_left < 2) a_vec[i].y = 0u;
                    if (sv_left < 3) a_vec[i].z = 0u;
                    if (sv_left < 4) a_vec[i].w = 0u;
                }
                if (in_tile) *(uint4*)&As[buf][a_lds0 + i * A_ROWSTEP * LDA] = a_vec[i];
            } else {
                if (in_tile) As[buf][a_lds0 + i * A_ROWSTEP * LDA] = a_sc[i];
            }
        }
#pragma unroll
        for (int j = 0; j < NCH; ++j) {
            if constexpr (CFG::B_KMAJOR) {
#pragma unroll
                for (int e = 0; e < CHW; ++e) {
                    elem_t x = b_reg[j][e];
                    if constexpr (SV) x = ((sv_keep >> (j * CHW + e)) & 1u) ? x : (elem_t)0;
                    Bs[buf][b_lds0 + (j * GROUPS * CHW + e) * LDB] = x;
                }
            } else {
                uint4 pk;
                pk.x = (uint32_t)b_reg[j][0] | ((uint32_t)b_reg[j][1] << 16);
                pk.y = (uint32_t)b_reg[j][2] | ((uint32_t)b_reg[j][3] << 16);
                pk.z = (uint32_t)b_reg[j][4] | ((uint32_t)b_reg[j][5] << 16);
                pk.w = (uint32_t)b_reg[j][6] | ((uint32_t)b_reg[j][7] << 16);
                *(uint4*)&Bs[buf][b_lds0 + j * GROUPS * CHW] = pk;
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

    const int fa_row0 = (wm * BM * MB + lrow) * LDA + kg * KPL;
    const int fb_col0 = wn * BN * MB + lrow;

    // Main loop.  A wave holds the operand fragments of step t in registers (fc); the tiles of step t+1 wait in the
    // staging registers.  It issues most MFMAs of step t, writes the staged tiles to the other LDS buffer, passes the
    // barrier, fetches the fragments of step t+1 (fn) and starts the global loads of step t+2 -- and only then issues
    // the last MFMAs of step t, which need nothing but registers: they cover the LDS latency and the barrier skew, so
    // the matrix pipe does not idle at the step boundary.
    constexpr int NU = igemm_units<CFG>();
    constexpr int TAILU = NU >= 4 ? NU / 4 : 1;
    auto body = [&](auto bufc, int step, IgemmFrags<CFG>& fc, IgemmFrags<CFG>& fn) {
        constexpr int buf = decltype(bufc)::value;
        const bool more = step + 1 < step_end;
        igemm_mma_range<CFG, 0, NU - TAILU>(fc, acc);
        if (more) store_tiles(std::integral_constant<int, buf ^ 1>{});
        __syncthreads();
        if (more) igemm_read_frags<CFG>(As[buf ^ 1], Bs[buf ^ 1], fn, fa_row0, fb_col0, kg);
        if (step + 2 < step_end) load_tiles(step + 2);
        __builtin_amdgcn_sched_barrier(0);  // keep the register-only MFMAs below behind the requests above
        igemm_mma_range<CFG, NU - TAILU, NU>(fc, acc);
    };

    if (step_begin < step_end) {
        IgemmFrags<CFG> f0, f1;
        load_tiles(step_begin);
        store_tiles(std::integral_constant<int, 0>{});
        __syncthreads();
        igemm_read_frags<CFG>(As[0], Bs[0], f0, fa_row0, fb_col0, kg);
        if (step_begin + 1 < step_end) load_tiles(step_begin + 1);
        for (int step = step_begin; step < step_end; step += 2) {
            body(std::integral_constant<int, 0>{}, step, f0, f1);
            if (step + 1 < step_end) body(std::integral_constant<int, 1>{}, step + 1, f1, f0);
        }
    }

    igemm_epilogue<CFG>(a, acc, p0, m0, wm, wn, lane, lrow);
}

// ---------------------------------------------------------------------------
// host side of a variant
// ---------------------------------------------------------------------------
template <class CFG, int PADMODE, bool SV = false>
hipError_t ugemm_launch(const Variant& v, ConvArgs& a, hipStream_t s)
{
    const int total_steps = ((SV ? a.QP : a.Q) + CFG::TK - 1) / CFG::TK;
    a.nsplit = v.split;
    a.steps_per_split = (total_steps + v.split - 1) / v.split;
    dim3 grid((unsigned)((a.P + CFG::TN - 1) / CFG::TN), (unsigned)((a.K + CFG::TM - 1) / CFG::TM), (unsigned)v.split);
    hipLaunchKernelGGL((ugemm_kernel<CFG, PADMODE, SV>), grid, dim3(CFG::NT), 0, s, a);
    return hipGetLastError();
}

template <class CFG, int PADMODE, bool SV = false>
bool ugemm_valid(const Variant& v, const conv_desc& d, int OH, int OW)
{
    if (d.dtype != CFG::DT) return false;
    const long long Q = (long long)d.C * d.R * d.S, P = (long long)d.N * OH * OW;
    if (SV && d.S < 3) return false;  // nothing to vectorise
    const long long ES = sizeof(typename CFG::elem_t);
    // 16-byte filter loads need 4-byte alignment only, so fp32 rows of any length qualify (the vector that straddles
    // the end of a row is fixed up word by word); 16-bit rows must be a multiple of the vector
    if (CFG::AVEC && ES == 2 && (Q % CFG::VEC) != 0) return false;
    if (PADMODE == PAD_NONE && d.pad != 0) return false;
    if (PADMODE == PAD_TAPS && (d.pad == 0 || d.R * d.S > 32)) return false;
    if (PADMODE == PAD_ROWCOL && (d.pad == 0 || d.R * d.S <= 32 || d.R > 16 || d.S > 16)) return false;
    // offsets are 32-bit sums of a vector part, a scalar part and the far markers: keep every tensor below 1 GiB
    const long long in_bytes = ((long long)d.N * d.C * d.H * d.W + (long long)d.pad * (d.W + 1)) * ES;
    if (in_bytes > kUgemmMaxBytes || (long long)d.K * Q * ES > kUgemmMaxBytes) return false;
    const int kcap = ((d.K + 31) / 32) * 32;
    if (CFG::TM > kcap && CFG::TM > 16) return false;
    if (CFG::TM == 96 && (d.K % 96) != 0) return false;
    const long long pcap = ((P + 63) / 64) * 64;
    if (CFG::TN > pcap) return false;
    const long long Qlay = SV ? (long long)d.C * d.R * ((d.S + 3) / 4 * 4) : Q;
    const long long steps = (Qlay + CFG::TK - 1) / CFG::TK;
    if (v.split > 1 && steps < 2LL * v.split) return false;
    if (v.split > 1 && (long long)d.K * P * 4 >= (1LL << 32)) return false;
    if (d.K > 65535LL * CFG::TM) return false;
    return true;
}

template <class CFG, int PADMODE, bool SV = false>
void ugemm_register_one(std::vector<Variant>& out, std::initializer_list<int> splits)
{
    for (int sk : splits) {
        Variant v;
        char buf[160];
        snprintf(buf, sizeof buf, "ug_%s_M%dN%dK%d_w%dx%d_b%d%s_%s%s", dtype_name(CFG::DT), CFG::TM, CFG::TN, CFG::TK, CFG::WM,
                 CFG::WN, CFG::MB, CFG::AVEC ? "_v" : "_s", PADMODE == PAD_NONE ? "p0" : PADMODE == PAD_TAPS ? "pt" : "prc",
                 SV ? "_s4" : "");
        v.name = buf;
        if (sk > 1) v.name += "_sk" + std::to_string(sk);
        v.dtype = CFG::DT;
        v.split = sk;
        v.tm = CFG::TM;
        v.tn = CFG::TN;
        v.tk = CFG::TK;
        v.threads = CFG::NT;
        v.family = FAM_IGEMM;
        v.specificity = 1 + (CFG::AVEC ? 1 : 0) + (SV ? 1 : 0);
        v.traits = TRAIT_REGISTER_OPERANDS | (CFG::AVEC ? 0u : TRAIT_SCALAR_LOADS) | (SV ? TRAIT_STRIDED_VECTOR : 0u);
        v.valid = &ugemm_valid<CFG, PADMODE, SV>;
        v.launch = &ugemm_launch<CFG, PADMODE, SV>;
        out.push_back(v);
    }
}

// one tile shape in all three padding modes (exactly one of them is valid for a given layer)
template <class CFG>
void ugemm_register(std::vector<Variant>& out, std::initializer_list<int> splits)
{
    ugemm_register_one<CFG, PAD_NONE>(out, splits);
    ugemm_register_one<CFG, PAD_TAPS>(out, splits);
    ugemm_register_one<CFG, PAD_ROWCOL>(out, splits);
}

// s-vector gather (four window columns per 16-byte load) for unpadded layers with wide windows
template <class CFG>
void ugemm_register_svec(std::vector<Variant>& out, std::initializer_list<int> splits)
{
    ugemm_register_one<CFG, PAD_NONE, true>(out, splits);
}

}  // namespace convfwd
