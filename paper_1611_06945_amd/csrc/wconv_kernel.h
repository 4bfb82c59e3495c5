// Window-reuse convolution for stride-1 layers on small images (fp32 MFMA).
//
// The paper's criticism of im2col + GEMM is that it does not reuse data between
// spatially overlapping windows and pays for a 4D -> 2D transform (Section 5,
// "Related Work").  This kernel answers both: a chunk of CB input channels of one
// image is copied once, untransformed, into LDS with its zero border, and all
// R*S taps of every output pixel are then read from that copy by adding a
// constant offset (r*PW + s) to the pixel's address.  There is no gather and no
// index arithmetic in the main loop: one LDS read per MFMA operand.
//
//   workgroup  = TM output channels x one image (x one tile of NB*16 pixels)
//   chunk      = CB = 16*CPL input channels: filter slab [TM][CB*R*S] (contiguous pieces of
//                KCRS rows) + padded image slab [CB][PH*PW] in LDS, double buffered
//   wave w, lane group g (16 lanes each) own channels (4w+g)*CPL .. +CPL of the chunk;
//   one MFMA 16x16x4 multiplies, for one tap, 16 output channels x 16 pixels x those 4 groups.
//   The four waves therefore hold partial sums over disjoint channels; they are added in a
//   fixed order through LDS at the end, then bias + activation are applied on the store.
#pragma once

#include <type_traits>

#include "igemm_kernel.h"

namespace convfwd {

template <int DT_, int R_, int S_, int CPL_, int TMB_, int NB_, int LB_, int WN_ = 2>
struct WconvCfg {
    static_assert(DT_ == CONV_F32, "fp32 only");
    static constexpr int DT = DT_, R = R_, S = S_, CPL = CPL_, TMB = TMB_, NB = NB_, LB = LB_, WN = WN_;
    static constexpr int NT = 256 * WN;          // 4 waves split the channels of a chunk, WN waves split the pixel blocks
    static constexpr int NBW = (NB + WN - 1) / WN;  // pixel blocks per wave (the last wave may own fewer)
    static constexpr int CB = 16 * CPL;        // channels per chunk
    static constexpr int TM = 16 * TMB;        // output channels per workgroup
    static constexpr int TNP = 16 * NB;        // pixel columns per workgroup
    static constexpr int KCH = CB * R * S;     // reduction elements per chunk
    static constexpr int LDA = KCH + 4;        // filter slab row pitch (floats)
    static constexpr CoopPlan planA = coop_plan(NT, TM * KCH / 4);
    static constexpr int RED_FLOATS = 4 * 16 * TNP;  // cross-wave reduction buffer, one 16-row block at a time
    static_assert((KCH % 4) == 0, "filter slab rows are moved as 16-byte vectors");

};

// Pitch of one channel plane of the padded image in LDS: the padded image, rounded up so that the planes of the four
// lane groups of a wave start 16 banks apart (their simultaneous reads then fall on different banks).
__host__ __device__ inline int wconv_plane(int H, int W, int pad)
{
    const int plane = (H + 2 * pad) * (W + 2 * pad);
    return plane + ((16 - plane % 64) + 64) % 64;
}

// Variants with one 16-row block per wave are meant to run two workgroups per CU (four waves per SIMD when the
// workgroup has 512 threads): the waves-per-SIMD attribute keeps the register allocation within that budget.
template <class CFG>
__global__ __launch_bounds__(CFG::NT) __attribute__((amdgpu_waves_per_eu(CFG::TMB == 1 ? CFG::NT / 128 : 1)))
void wconv_kernel(ConvArgs a)
{
    constexpr int R = CFG::R, S = CFG::S, RS = R * S, CPL = CFG::CPL, TMB = CFG::TMB, NB = CFG::NB, CB = CFG::CB;
    constexpr int TM = CFG::TM, TNP = CFG::TNP, KCH = CFG::KCH, LDA = CFG::LDA, NT = CFG::NT, LB = CFG::LB, NBW = CFG::NBW;
    constexpr CoopPlan planA = CFG::planA;
    extern __shared__ __attribute__((aligned(16))) float smem[];

    const int PW = a.W + 2 * a.pad, PLANE = wconv_plane(a.H, a.W, a.pad);
    float* const As0 = smem;                         // [2][TM*LDA]
    float* const Bs0 = smem + 2 * TM * LDA;          // [2][CB*PLANE]
    const int b_elems = CB * PLANE;

    const int tid = threadIdx.x, lane = tid & 63, li = lane & 15, g = lane >> 4;
    // wave-uniform by construction; saying so keeps the per-wave decisions below on the scalar unit
    const int w = __builtin_amdgcn_readfirstlane((tid >> 6) & 3), wn = __builtin_amdgcn_readfirstlane(tid >> 8);
    const int nb0 = wn * NBW;  // first pixel block of this wave
    const int ntiles = (a.OHW + TNP - 1) / TNP;
    const int img = blockIdx.x / ntiles, ntile = blockIdx.x - img * ntiles;
    const int m0 = blockIdx.y * TM;
    const int n0 = ntile * TNP;

    const int total_chunks = a.C / CB;
    const int chunk_begin = blockIdx.z * a.steps_per_split;
    int chunk_end = chunk_begin + a.steps_per_split;
    if (chunk_end > total_chunks) chunk_end = total_chunks;

    const __amdgpu_buffer_rsrc_t rin = make_rsrc(a.in, a.in_bytes);
    const __amdgpu_buffer_rsrc_t rfilt = make_rsrc(a.filt, a.filt_bytes);

    const int nvecB = (CB * a.HW) >> 2;  // 16-byte vectors of one image slab in global memory

    uint4 a_reg[planA.loads];
    uint4 b_reg[LB];

    auto load_chunk = [&](int chunk) {
        const int c0 = chunk * CB;
#pragma unroll
        for (int i = 0; i < planA.loads; ++i) {
            const int v = i * NT + tid;
            const bool in_tile = (i + 1 < planA.loads || !planA.last_guarded) ? true : (v < TM * KCH / 4);
            const int row = v / (KCH / 4), col = (v % (KCH / 4)) * 4;
            const bool ok = in_tile && (m0 + row < a.K);
            a_reg[i] = buffer_load_vec(rfilt, ok ? (uint32_t)((m0 + row) * a.Q + c0 * RS + col) * 4u : kOutOfRange);
        }
        const uint32_t slab = (uint32_t)((img * a.C + c0) * a.HW) * 4u;
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            const int v = i * NT + tid;
            b_reg[i] = buffer_load_vec(rin, v < nvecB ? slab + (uint32_t)v * 16u : kOutOfRange);
        }
    };

    // the first chunk's loads go out before anything else: their latency is covered by the set-up work below
    if (chunk_begin < chunk_end) load_chunk(chunk_begin);

    // zero both image slabs once: the border stays zero, the interior is overwritten by every chunk
    for (int i = tid; i < 2 * b_elems; i += NT) Bs0[i] = 0.0f;

    // Where each element this thread moves lands in the padded LDS slab.  The same for every chunk, so the
    // divisions are done once here and the main loop only adds the buffer base (-1: nothing to move).
    int b_idx[LB][4];
#pragma unroll
    for (int i = 0; i < LB; ++i) {
        const int v = i * NT + tid;
        // the vector's first element by division, the other three by stepping (x, y, channel) with carries
        uint32_t cl, pix, y, x;
        a.dHW.divmod((uint32_t)(4 * v), cl, pix);
        a.dW.divmod(pix, y, x);
        int ci = (int)cl, yi = (int)y, xi = (int)x;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            b_idx[i][e] = v < nvecB ? ci * PLANE + (yi + a.pad) * PW + xi + a.pad : -1;
            if (++xi == a.W) {
                xi = 0;
                if (++yi == a.H) {
                    yi = 0;
                    ++ci;
                }
            }
        }
    }

    auto store_chunk = [&](int buf) {
        float* As = As0 + buf * TM * LDA;
        float* Bs = Bs0 + buf * b_elems;  // buf is a constant at every call site: LDS addresses are base + immediate
#pragma unroll
        for (int i = 0; i < planA.loads; ++i) {
            const int v = i * NT + tid;
            const bool in_tile = (i + 1 < planA.loads || !planA.last_guarded) ? true : (v < TM * KCH / 4);
            const int row = v / (KCH / 4), col = (v % (KCH / 4)) * 4;
            if (in_tile) *(uint4*)&As[row * LDA + col] = a_reg[i];
        }
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            if (b_idx[i][0] >= 0) {
                const uint32_t vals[4] = {b_reg[i].x, b_reg[i].y, b_reg[i].z, b_reg[i].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) Bs[b_idx[i][e]] = __builtin_bit_cast(float, vals[e]);
            }
        }
    };

    // address (inside one channel plane) of the window's first element, for each pixel column of this lane
    int bpos[NBW];
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb) {
        const int n = n0 + (nb0 + nb) * 16 + li;
        uint32_t oy, ox;
        a.dOW.divmod(n < a.OHW ? (uint32_t)n : 0u, oy, ox);
        bpos[nb] = (int)oy * PW + (int)ox;
    }
    const int chan0 = (w * 4 + g) * CPL;

    f32x4 acc[TMB][NBW];
#pragma unroll
    for (int mb = 0; mb < TMB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb) acc[mb][nb] = f32x4{0.f, 0.f, 0.f, 0.f};
    const bool last_block_real = nb0 + NBW <= NB;  // wave-uniform: false when NB is not a multiple of WN

    // taps [T0, T1) of the chunk (a tap = one channel of the lane group x one window position)
    auto compute = [&](int buf, auto t0, auto t1) {
        constexpr int T0 = decltype(t0)::value, T1 = decltype(t1)::value;
        const float* __restrict__ As = As0 + buf * TM * LDA + li * LDA + chan0 * RS;
        const float* __restrict__ Bs = Bs0 + buf * b_elems + chan0 * PLANE;
        // operands of tap t+1 are requested from LDS before the MFMAs of tap t are issued
        float av[2][TMB], bv[2][NBW];
        auto fetch = [&](int t, int slot) {
            const int cc = t / RS, r = (t % RS) / S, s = t % S;
#pragma unroll
            for (int mb = 0; mb < TMB; ++mb) av[slot][mb] = As[mb * 16 * LDA + t];
            const int toff = cc * PLANE + r * PW + s;
#pragma unroll
            for (int nb = 0; nb < NBW; ++nb) bv[slot][nb] = Bs[bpos[nb] + toff];
        };
        if (T0 < T1) fetch(T0, T0 & 1);
#pragma unroll
        for (int t = T0; t < T1; ++t) {
            if (t + 1 < T1) fetch(t + 1, (t + 1) & 1);
#pragma unroll
            for (int mb = 0; mb < TMB; ++mb)
#pragma unroll
                for (int nb = 0; nb < NBW; ++nb)
                    if (nb + 1 < NBW || last_block_real)
                        acc[mb][nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[t & 1][mb], bv[t & 1][nb], acc[mb][nb], 0, 0, 0);
        }
    };
    constexpr int TAPS = CPL * RS;
    constexpr int TSPLIT = (TAPS * 5 + 8) / 9;  // the next chunk is written to LDS after this many taps
    typedef std::integral_constant<int, 0> tap_first;
    typedef std::integral_constant<int, TSPLIT> tap_mid;
    typedef std::integral_constant<int, TAPS> tap_last;

    // One chunk on LDS buffer `buf` (a compile-time constant: the loop below is unrolled by two, so every LDS address
    // is a per-thread base plus an immediate and no vector instruction is spent on buffer switching -- on this device
    // vector-ALU instructions and fp32 MFMAs of a SIMD never overlap).  The other LDS buffer was last read before the
    // barrier that ended the previous chunk, so the next chunk is written into it in the middle of this chunk's MFMA
    // chain: the LDS writes then overlap the matrix pipe instead of following it.
    auto body = [&](auto bufc, int chunk) {
        constexpr int buf = decltype(bufc)::value;
        const bool more = chunk + 1 < chunk_end;
        if (more) load_chunk(chunk + 1);
        compute(buf, tap_first{}, tap_mid{});
        if (more) store_chunk(buf ^ 1);
        compute(buf, tap_mid{}, tap_last{});
        __syncthreads();
    };
    if (chunk_begin < chunk_end) {
        __syncthreads();  // zero fill done before the first interior write
        store_chunk(0);
        __syncthreads();
        for (int chunk = chunk_begin; chunk < chunk_end; chunk += 2) {
            body(std::integral_constant<int, 0>{}, chunk);
            if (chunk + 1 < chunk_end) body(std::integral_constant<int, 1>{}, chunk + 1);
        }
    } else {
        __syncthreads();
    }

    // ---- add the four waves' partial sums in wave order, then bias + activation + store ------------
    float* const red = smem;  // [4 waves][16 rows][TNP]
    const bool split = a.nsplit > 1;
    const __amdgpu_buffer_rsrc_t rbias = make_rsrc(a.bias, a.bias ? (uint32_t)a.K * 4u : 0u);
    const __amdgpu_buffer_rsrc_t rout = make_rsrc(a.out, a.out_bytes);
    const __amdgpu_buffer_rsrc_t rws = make_rsrc(a.ws + (size_t)blockIdx.z * a.K * a.P, (uint32_t)a.K * a.P * 4u);
#pragma unroll
    for (int mb = 0; mb < TMB; ++mb) {
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb)
            if (nb + 1 < NBW || last_block_real) {
#pragma unroll
                for (int v = 0; v < 4; ++v) red[(w * 16 + 4 * g + v) * TNP + (nb0 + nb) * 16 + li] = acc[mb][nb][v];
            }
        __syncthreads();
        if (a.pool) {
            // the tile is the whole image: 3x3 stride-2 maxima of the summed block, then bias + activation (both
            // monotone, so this equals pooling the activations)
            const int npool = a.POH * a.POW;
            for (int e = tid; e < 16 * npool; e += NT) {
                uint32_t urow, upp, upy, upx;  // a.dX divides by POH*POW, a.dY by POW
                a.dX.divmod((uint32_t)e, urow, upp);
                a.dY.divmod(upp, upy, upx);
                const int row = (int)urow, pp = (int)upp, py = (int)upy, px = (int)upx;
                const int k = m0 + mb * 16 + row;
                float m = -INFINITY;
#pragma unroll
                for (int dy = 0; dy < 3; ++dy)
#pragma unroll
                    for (int dx = 0; dx < 3; ++dx) {
                        const int idx = row * TNP + (2 * py + dy) * a.OW + 2 * px + dx;
                        float x = red[idx];
                        x += red[16 * TNP + idx];
                        x += red[32 * TNP + idx];
                        x += red[48 * TNP + idx];
                        m = (x > m || (!a.relu && x != x)) ? x : m;  // NaN: dropped by the activation, else it is the result
                    }
                const bool ok = k < a.K;
                m += buffer_load_elem<float>(rbias, ok ? (uint32_t)k * 4u : kOutOfRange);
                if (a.relu) m = m > 0.0f ? m : 0.0f;
                buffer_store_elem<float>(m, rout, ok ? (uint32_t)((img * a.K + k) * npool + pp) * 4u : kOutOfRange);
            }
            __syncthreads();
            continue;
        }
        constexpr int NE = (16 * TNP + NT - 1) / NT;  // outputs of this 16-row block per thread
        // element j*NT + tid of the [16][TNP] block: row and column by one division, then by stepping
        int rowj[NE], colj[NE];
        {
            int row = tid / TNP, col = tid - row * TNP;
#pragma unroll
            for (int j = 0; j < NE; ++j) {
                rowj[j] = row;
                colj[j] = col;
                row += NT / TNP;
                col += NT % TNP;
                if (col >= TNP) {
                    col -= TNP;
                    ++row;
                }
            }
        }
        float bs[NE];
#pragma unroll
        for (int j = 0; j < NE; ++j) {  // all bias values first: one round trip instead of one per output
            const bool in_block = ((j + 1) * NT <= 16 * TNP) ? true : (j * NT + tid < 16 * TNP);
            bs[j] = buffer_load_elem<float>(rbias, (in_block && !split) ? (uint32_t)(m0 + mb * 16 + rowj[j]) * 4u : kOutOfRange);
        }
#pragma unroll
        for (int j = 0; j < NE; ++j) {
            const bool in_block = ((j + 1) * NT <= 16 * TNP) ? true : (j * NT + tid < 16 * TNP);
            const int idx = in_block ? j * NT + tid : 0;
            float x = red[idx];
            x += red[16 * TNP + idx];
            x += red[32 * TNP + idx];
            x += red[48 * TNP + idx];
            const int k = m0 + mb * 16 + rowj[j], n = n0 + colj[j];
            const bool ok = in_block && k < a.K && n < a.OHW;
            if (split) {
                buffer_store_elem<float>(x, rws, ok ? (uint32_t)(k * a.P + img * a.OHW + n) * 4u : kOutOfRange);
            } else {
                x += bs[j];
                if (a.relu) x = x > 0.0f ? x : 0.0f;
                buffer_store_elem<float>(x, rout, ok ? (uint32_t)((img * a.K + k) * a.OHW + n) * 4u : kOutOfRange);
            }
        }
        __syncthreads();
    }
}

template <class CFG>
size_t wconv_lds_bytes(int H, int W, int pad)
{
    const size_t plane = (size_t)wconv_plane(H, W, pad);
    const size_t pipe = 2 * ((size_t)CFG::TM * CFG::LDA + (size_t)CFG::CB * plane);
    return sizeof(float) * (pipe > (size_t)CFG::RED_FLOATS ? pipe : (size_t)CFG::RED_FLOATS);
}

template <class CFG>
hipError_t wconv_launch(const Variant& v, ConvArgs& a, hipStream_t s)
{
    const size_t lds = wconv_lds_bytes<CFG>(a.H, a.W, a.pad);
    const hipError_t e = ensure_dynamic_lds((const void*)wconv_kernel<CFG>, lds);
    if (e != hipSuccess) return e;
    const int total_chunks = a.C / CFG::CB;
    a.nsplit = v.split;
    a.steps_per_split = (total_chunks + v.split - 1) / v.split;
    const int ntiles = (a.OHW + CFG::TNP - 1) / CFG::TNP;
    dim3 grid((unsigned)(a.N * ntiles), (unsigned)((a.K + CFG::TM - 1) / CFG::TM), (unsigned)v.split);
    if (a.pool) {
        a.dX = make_fastdiv((uint32_t)(a.POH * a.POW));
        a.dY = make_fastdiv((uint32_t)a.POW);
    }
    hipLaunchKernelGGL(wconv_kernel<CFG>, grid, dim3(CFG::NT), lds, s, a);
    return hipGetLastError();
}

template <class CFG>
bool wconv_valid(const Variant& v, const conv_desc& d, int OH, int OW)
{
    if (d.dtype != CFG::DT || d.R != CFG::R || d.S != CFG::S || d.stride != 1) return false;
    if ((d.C % CFG::CB) != 0) return false;
    const long long HW = (long long)d.H * d.W, OHW = (long long)OH * OW;
    if ((long long)CFG::CB * HW / 4 > (long long)CFG::NT * CFG::LB) return false;  // image slab must fit the loader
    if (wconv_lds_bytes<CFG>(d.H, d.W, d.pad) > 160 * 1024) return false;
    const long long ntiles = (OHW + CFG::TNP - 1) / CFG::TNP;
    if (OHW * 10 < ntiles * CFG::TNP * 7) return false;  // at least 70 % of the pixel columns must be real
    if (ntiles > 1 && CFG::LB <= 4 && CFG::NB > 8) return false;  // small-image variants tile the pixels only with their small tiles
    const int chunks = d.C / CFG::CB;
    if (v.split > 1 && chunks < 2 * v.split) return false;
    const long long P = (long long)d.N * OHW;
    if (v.split > 1 && (long long)d.K * P * 4 >= (1LL << 32)) return false;
    if (CFG::TM > 16 && d.K < CFG::TM) return false;
    if (d.K > 65535LL * CFG::TM || (long long)d.N * ntiles > 2147483647LL) return false;
    // the fused max-pool reads its windows from the workgroup's own tile: the whole image, no partial sums elsewhere
    if ((d.flags & CONV_FLAG_MAXPOOL_3X3S2) && (ntiles != 1 || v.split > 1)) return false;
    return true;
}

template <class CFG>
void wconv_register(std::vector<Variant>& out, std::initializer_list<int> splits)
{
    for (int sk : splits) {
        Variant v;
        char buf[160];
        snprintf(buf, sizeof buf, "wconv_%s_%dx%d_M%dN%dC%d_w4x%d", dtype_name(CFG::DT), CFG::R, CFG::S, CFG::TM,
                 CFG::TNP, CFG::CB, CFG::WN);
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
        v.traits = TRAIT_POOL_EPILOGUE;
        v.valid = &wconv_valid<CFG>;
        v.launch = &wconv_launch<CFG>;
        out.push_back(v);
    }
}

}  // namespace convfwd
