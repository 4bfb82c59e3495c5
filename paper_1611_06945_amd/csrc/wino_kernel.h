// Winograd F(2x2, 3x3) convolution for 3x3 stride-1 layers, fp32 (16x16x4 MFMA).
//
// The paper names Winograd convolution as what makes the vendor library faster than its own kernels on 3x3 layers
// and as the main topic it leaves open (Section 4, "Experimental Results"; Section 5, "Related Work").  The minimal
// filtering algorithm F(2x2, 3x3) computes a 2x2 block of outputs from a 4x4 input tile d and a 3x3 filter g as
//     Y = A^T [ (G g G^T) .* (B^T d B) ] A
// and, summed over input channels, the element-wise product becomes 16 independent small matrix products
//     M[xi][k][t] = sum_c U[xi][k][c] * V[xi][c][t],    xi = 0..15, t = tile index over (image, tile row, tile column)
// with 2.25 times fewer multiplications than the direct form.  On this GPU the fp32 MFMA rate is what bounds the direct
// kernels while the vector ALU, LDS and L2 have slack, so the transforms are done inside the product kernel:
//   * U = G g G^T is computed once per call by a small kernel into the workspace, laid out so that a lane's MFMA
//     operands of one step are one contiguous 8- or 16-byte load.  Every plane xi belongs to exactly one wave, so the
//     transformed filters go from global memory straight into that wave's registers: no LDS staging;
//   * a workgroup owns TM output channels x TT consecutive tiles and walks the input channels CB at a time.  Per step
//     the input rows its tiles touch are copied into LDS with their zero border (coalesced loads, the positions are the
//     same in every step), each (tile, channel) is transformed by one thread (32 additions) into V[xi][channel][tile],
//     and every wave multiplies its share of the 16 xi planes: per plane MBLK x NBLK blocks of 16x16, CB/4 MFMAs each;
//   * at the end the 16 planes meet in LDS, each (channel, tile) is transformed back by one thread (24 additions) and
//     its 2x2 outputs leave with bias and activation applied.
// Every sum is taken in a fixed order: results are bit-reproducible.  Products of small integers stay exact (the
// filter transform only halves), so integer-valued tests match the direct definition bit for bit.
#pragma once

#include <type_traits>

#include "igemm_kernel.h"

namespace convfwd {

struct WinoF3 {  // what a 12-byte buffer load returns (the vector type is padded to 16 bytes)
    float x, y, z, unused;
};

template <int MBLK_, int NBLK_, int XW_, int LBE_, int CB_, int FF_ = 0>
struct WinoCfg {
    static constexpr int MBLK = MBLK_, NBLK = NBLK_, XW = XW_, LBE = LBE_, CB = CB_;
    // FF: the filter transform runs inside the product kernel, step by step (no filter kernel, no workspace)
    static constexpr bool FF = FF_ != 0;
    static constexpr int WAVES = 16 / XW;        // every wave owns XW of the 16 transform planes
    static constexpr int NT = 64 * WAVES;
    static constexpr int TM = 16 * MBLK;         // output channels per workgroup
    static constexpr int TT = 16 * NBLK;         // tiles (2x2 output blocks) per workgroup
    static constexpr int HN = CB / 4;            // MFMAs per block and step (4 channels each)
    // The transformed tiles are [16 planes][CB channels][tiles] in LDS: the 16 lanes that feed one channel of an MFMA
    // read 16 consecutive floats, and the pitch is 16 mod 32 so that the four channel groups of a wave use different banks
    static constexpr int VP = TT + (TT % 32 == 0 ? 16 : 0);
    static constexpr int V_FLOATS = 16 * CB * VP;  // one buffer of transformed tiles
    static constexpr int MP = TT + 4;            // row pitch of the plane buffer of the epilogue (4 mod 8: conflict-free writes)
    // FF: transformed filters of a step in LDS, [16 planes][4 lane groups][TM channels][HN]; the group pitch is 8 mod 32
    // floats so that the transform's 8 writes of one filter row (4 groups x 2) fall on different banks
    static constexpr int UQ = TM * HN + 8;
    static constexpr int U_FLOATS = FF ? 16 * 4 * UQ : 0;
    static_assert(!FF || (CB == 8 && TM * CB <= NT), "one filter per thread and step");
    static_assert(16 % XW == 0 && (CB == 8 || CB == 16) && TT * CB <= NT, "one transform task per thread");
};

struct WinoGeom {
    int TH, TW;      // tiles per image column / row
    int tiles_img;   // TH * TW
    int tiles;       // N * tiles_img
    int nr_max;      // tile rows (of any images) one workgroup's tiles can touch
    int PWL;         // floats per staged input row: 2*TW + 2 (even)
    int raw_chan;    // floats per channel of the staged rows: nr_max * 4 * PWL, padded to 4 mod 32
};

template <class CFG>
__host__ __device__ inline WinoGeom wino_geom(int N, int OH, int OW)
{
    WinoGeom g;
    g.TH = (OH + 1) / 2;
    g.TW = (OW + 1) / 2;
    g.tiles_img = g.TH * g.TW;
    g.tiles = N * g.tiles_img;
    g.nr_max = (CFG::TT + g.TW - 2) / g.TW + 1;
    g.PWL = 2 * g.TW + 2;
    g.raw_chan = g.nr_max * 4 * g.PWL;
    g.raw_chan += ((4 - g.raw_chan % 32) + 32) % 32;
    return g;
}

template <class CFG>
size_t wino_lds_bytes(int N, int OH, int OW)
{
    const WinoGeom g = wino_geom<CFG>(N, OH, OW);
    const size_t pipe = sizeof(float) * (2 * (size_t)CFG::V_FLOATS + 2 * (size_t)CFG::CB * g.raw_chan + 2 * (size_t)CFG::U_FLOATS);
    const size_t epi = sizeof(float) * 16 * (size_t)CFG::TM * CFG::MP;
    return pipe > epi ? pipe : epi;
}

__host__ __device__ inline int wino_kpitch(int K) { return (K + 3) & ~3; }

// ConvArgs::dX, dY, dZ carry the divisions by TW, TH and TH*TW for this family.

// Filter transform.  With HN = CB/4 and K' = wino_kpitch(K), the workspace holds
//     U[c / CB][xi][q][k][h] = (G g G^T)[xi / 4][xi % 4] of filter (k, c),   c % CB = q + 4*h,  q = 0..3, h = 0..HN-1
// (G = [1 0 0; 1/2 1/2 1/2; 1/2 -1/2 1/2; 0 0 1]): MFMA lane group q of a wave consumes channel q + 4*h in its h-th MFMA
// of a step, so the HN values it needs for one output channel are adjacent.  A workgroup transforms 32 x CB filters,
// one per thread: their values are read as contiguous runs into LDS, all loads in flight at once, and the threads are
// ordered (h, k, q) so that a wave's stores of one plane are one contiguous run.
template <int CB>
__global__ __launch_bounds__(32 * CB) void wino_filter_kernel(const float* __restrict__ filt, float* __restrict__ U, int K, int C)
{
    // one thread per filter (k, c): thread = h + HN*kl + 32*HN*q, so that a wave's stores of one plane are one contiguous run
    constexpr int HN = CB / 4, ROW = CB * 9 + 1;  // odd row pitch: the lanes' strided reads fall on different banks
    constexpr int NTH = 32 * CB;
    constexpr int NLOAD = 32 * CB * 9 / NTH;
    __shared__ float g_s[32 * ROW];
    const int tid = threadIdx.x;
    const int k0 = blockIdx.x * 32, cb = blockIdx.y;
    float v[NLOAD];
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
        const int e = i * NTH + tid;
        const int kl = e / (CB * 9), j = e - kl * (CB * 9);
        v[i] = (k0 + kl < K) ? filt[((size_t)(k0 + kl) * C + cb * CB) * 9 + j] : 0.0f;
    }
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
        const int e = i * NTH + tid;
        const int kl = e / (CB * 9), j = e - kl * (CB * 9);
        g_s[kl * ROW + j] = v[i];
    }
    __syncthreads();
    const int h = tid % HN, kl = (tid / HN) & 31, q = tid / (32 * HN);
    if (k0 + kl >= K) return;
    const size_t kp = (size_t)wino_kpitch(K);
    float u[16];
    {
        const float* g = g_s + kl * ROW + (q + 4 * h) * 9;
        float gg[4][3];
#pragma unroll
        for (int j = 0; j < 3; ++j) {
            const float g0 = g[j], g1 = g[3 + j], g2 = g[6 + j];
            gg[0][j] = g0;
            gg[1][j] = 0.5f * ((g0 + g2) + g1);
            gg[2][j] = 0.5f * ((g0 + g2) - g1);
            gg[3][j] = g2;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float a0 = gg[i][0], a1 = gg[i][1], a2 = gg[i][2];
            u[4 * i + 0] = a0;
            u[4 * i + 1] = 0.5f * ((a0 + a2) + a1);
            u[4 * i + 2] = 0.5f * ((a0 + a2) - a1);
            u[4 * i + 3] = a2;
        }
    }
    float* dst = U + (((size_t)cb * 16 * 4 + q) * kp + k0 + kl) * HN + h;
    const size_t plane = 4 * kp * HN;
#pragma unroll
    for (int xi = 0; xi < 16; ++xi) dst[xi * plane] = u[xi];
}

template <class CFG>
__global__ __launch_bounds__(CFG::NT) void wino_kernel(ConvArgs a)
{
    constexpr int MBLK = CFG::MBLK, NBLK = CFG::NBLK, XW = CFG::XW, LBE = CFG::LBE, NT = CFG::NT, TM = CFG::TM, TT = CFG::TT;
    constexpr int CB = CFG::CB, HN = CFG::HN, V_FLOATS = CFG::V_FLOATS, MP = CFG::MP, VP = CFG::VP;
    constexpr bool FF = CFG::FF;
    constexpr int UQ = CFG::UQ, U_FLOATS = CFG::U_FLOATS;
    constexpr uint32_t kFar = 0x80000000u;  // tensors stay below 2 GiB: this offset plus any in-range scalar offset is out of range
    typedef Mma<CONV_F32, 16> mma_t;
    extern __shared__ __attribute__((aligned(16))) float smem[];

    const WinoGeom geo = wino_geom<CFG>(a.N, a.OH, a.OW);
    const int PWL = geo.PWL, raw_chan = geo.raw_chan;
    float* const Vs0 = smem;                      // [2][16][CB][VP]
    float* const Rs0 = Vs0 + 2 * V_FLOATS;        // [2][CB][raw_chan]: rows [nr_max][4][PWL] per channel
    float* const Us0 = Rs0 + 2 * CB * raw_chan;   // FF: [2][16][4][UQ]

    const int tid = threadIdx.x, lane = tid & 63, li = lane & 15, kq = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Workgroup -> (channel tile, tile group).  Workgroups are dealt round-robin to the 8 XCDs, each with its own L2, so the
    // ids an XCD receives (id % 8 fixed) are mapped to one contiguous run of the order "groups of 3 channel tiles; within a
    // group all tile groups; within a tile group the 3 channel tiles": an XCD then touches about 3 channel tiles of the
    // transformed filters and an eighth-to-a-quarter of the images instead of everything.
    int t0, m0;
    {
        const int KT = (a.K + TM - 1) / TM, TN = (geo.tiles + TT - 1) / TT, total = KT * TN;
        const int x = blockIdx.x & 7, j = blockIdx.x >> 3;
        const int s = x * (total >> 3) + (x < (total & 7) ? x : (total & 7)) + j;  // runs in XCD order, sized as the hardware deals them
        const int per_group = 3 * TN;
        const int g = s / per_group, rem = s - g * per_group;
        const int gs = (KT - 3 * g) < 3 ? (KT - 3 * g) : 3;
        const int tg = rem / gs, kk = rem - tg * gs;
        t0 = tg * TT;
        m0 = (3 * g + kk) * TM;
    }
    const int chunks = a.C / CB;

    const __amdgpu_buffer_rsrc_t rin = make_rsrc(a.in, a.in_bytes);
    const int kp = wino_kpitch(a.K);
    const __amdgpu_buffer_rsrc_t ru = make_rsrc(a.ws, (uint32_t)kp * (uint32_t)a.C * 64u);

    // ---- transformed filters: lane (li, kq) of the wave that owns plane xi loads U[step][xi][kq][m0 + mb*16 + li][0..HN) ----
    const uint32_t u_off = (uint32_t)(((wave * XW * 4 + kq) * kp + m0 + li) * HN) * 4u;
    const uint32_t u_plane = (uint32_t)(4 * kp * HN) * 4u;   // bytes between two planes
    const uint32_t u_step = (uint32_t)kp * (uint32_t)(64 * CB);  // bytes between two steps

    // ---- input rows: the tile rows g_first .. g_last (index n*TH + ty) each need 4 input rows; element = (row, x) ----
    uint32_t g_first, t_in_row;
    a.dX.divmod((uint32_t)t0, g_first, t_in_row);
    const int t_last = (t0 + TT < geo.tiles ? t0 + TT : geo.tiles) - 1;
    const int nrows = ((int)a.dX.div((uint32_t)t_last) - (int)g_first + 1) * 4;
    uint32_t r_goff[LBE];
    int r_lds[LBE];
#pragma unroll
    for (int i = 0; i < LBE; ++i) {
        const int e = i * NT + tid;
        uint32_t ri, x, n, ty;
        a.dW.divmod((uint32_t)e, ri, x);
        const bool in_rows = (int)ri < nrows;
        a.dY.divmod(g_first + (in_rows ? (ri >> 2) : 0u), n, ty);
        const int y = 2 * (int)ty - a.pad + (int)(ri & 3u);
        const bool ok = in_rows && (unsigned)y < (unsigned)a.H;
        r_goff[i] = ok ? (uint32_t)(((int)n * a.C * a.H + y) * a.W + (int)x) * 4u : kFar;
        r_lds[i] = ok ? (int)ri * PWL + (int)x + a.pad : -1;
    }
    const uint32_t chan_bytes = (uint32_t)a.HW * 4u;

    // Register sets are named by step parity.  Filter fragments of step j are loaded at the top of step j - 1; the input
    // rows of step j are loaded at the top of step j - 3 and written to LDS in step j - 2 (transformed in step j - 1).
    // All loads in the loop are unconditional: past the last step they fall outside the tensors (and read as zero) or on
    // data that is never used.  A conditional load would force every later wait to assume it was skipped, i.e. to wait
    // for everything in flight.
    float af[2][XW][MBLK][HN], bf[2][XW][NBLK][HN];
    float r_reg[2][LBE][CB];

    auto load_filters = [&](auto setc, int chunk) {
        constexpr int set = decltype(setc)::value;
        if constexpr (FF) return;
        const uint32_t soff = (uint32_t)chunk * u_step;
#pragma unroll
        for (int x = 0; x < XW; ++x)
#pragma unroll
            for (int mb = 0; mb < MBLK; ++mb) {
                const uint32_t off = u_off + (uint32_t)x * u_plane + (uint32_t)(mb * 16 * HN) * 4u;
                if constexpr (HN == 2) {
                    const float2 t = __builtin_bit_cast(float2, __builtin_amdgcn_raw_buffer_load_b64(ru, (int)off, (int)soff, 0));
                    af[set][x][mb][0] = t.x;
                    af[set][x][mb][1] = t.y;
                } else {
                    // (the whole vector is cast at once: a bit cast of a single vector element reads element 0)
                    const float4 t = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(ru, (int)off, (int)soff, 0));
                    af[set][x][mb][0] = t.x;
                    af[set][x][mb][1] = t.y;
                    af[set][x][mb][2] = t.z;
                    af[set][x][mb][3] = t.w;
                }
            }
    };
    // FF: filter task (kl, cl) = (t / CB, t % CB) owns filter (m0 + kl, chunk*CB + cl) of every step: its 9 taps are 36
    // contiguous bytes, the CB filters of one output channel 36*CB contiguous bytes.  They are loaded two steps ahead,
    // transformed one step ahead
    // and written to LDS in the layout the MFMA lanes read: plane, lane group q = cl % 4, channel, h = cl / 4.
    const __amdgpu_buffer_rsrc_t rf = make_rsrc(a.filt, a.filt_bytes);
    // the filter tasks take the threads from the top of the workgroup, the input-transform tasks those from the bottom: the
    // waves that do both are as few as possible
    const int f_t = tid - (NT - TM * CB);
    const bool f_task = FF && f_t >= 0;
    const int f_kl = (f_t >= 0 ? f_t : 0) / CB, f_cl = (f_t >= 0 ? f_t : 0) % CB;
    const uint32_t f_off = (f_task && m0 + f_kl < a.K) ? (uint32_t)(((m0 + f_kl) * a.C + f_cl) * 9) * 4u : kFar;
    const int f_dst = (f_cl & 3) * UQ + f_kl * HN + (f_cl >> 2);
    float fr[2][FF ? 9 : 1];
    auto load_raw = [&](auto setc, int chunk) {
        constexpr int set = decltype(setc)::value;
        if constexpr (FF) {
            const uint32_t soff = (uint32_t)(chunk * CB * 9) * 4u;
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                const WinoF3 t = __builtin_bit_cast(WinoF3, __builtin_amdgcn_raw_buffer_load_b96(rf, (int)(f_off + 12u * j), (int)soff, 0));
                fr[set][3 * j + 0] = t.x;
                fr[set][3 * j + 1] = t.y;
                fr[set][3 * j + 2] = t.z;
            }
        }
    };
    auto transform_filters = [&](auto setc, auto bufc) {
        constexpr int set = decltype(setc)::value, buf = decltype(bufc)::value;
        if constexpr (FF) {
            if (f_task) {
                // G g G^T with the halves folded into fused multiply-adds: (a0 + a2 +- a1) / 2 = fma(a0 + a2, 1/2, +- a1 / 2)
                // (4 operations per column or row instead of 5; exact whenever the direct form is, e.g. on small integers)
                const float* g = fr[set];
                float gg[4][3];
#pragma unroll
                for (int j = 0; j < 3; ++j) {
                    const float g0 = g[j], g1 = g[3 + j], g2 = g[6 + j];
                    const float t = g0 + g2, hg = 0.5f * g1;
                    gg[0][j] = g0;
                    gg[1][j] = __builtin_fmaf(t, 0.5f, hg);
                    gg[2][j] = __builtin_fmaf(t, 0.5f, -hg);
                    gg[3][j] = g2;
                }
                float* Us = Us0 + buf * U_FLOATS + f_dst;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float a0 = gg[i][0], a1 = gg[i][1], a2 = gg[i][2];
                    const float t = a0 + a2, ha = 0.5f * a1;
                    Us[(4 * i + 0) * 4 * UQ] = a0;
                    Us[(4 * i + 1) * 4 * UQ] = __builtin_fmaf(t, 0.5f, ha);
                    Us[(4 * i + 2) * 4 * UQ] = __builtin_fmaf(t, 0.5f, -ha);
                    Us[(4 * i + 3) * 4 * UQ] = a2;
                }
            }
        }
    };
    auto read_filters = [&](auto bufc) {  // FF: this wave's planes, lane (li, kq): channels m0 + mb*16 + li, h = 0..HN-1
        constexpr int buf = decltype(bufc)::value;
        if constexpr (FF) {
            const float* Us = Us0 + buf * U_FLOATS + ((wave * XW) * 4 + kq) * UQ + li * HN;
#pragma unroll
            for (int x = 0; x < XW; ++x)
#pragma unroll
                for (int mb = 0; mb < MBLK; ++mb) {
                    const float2 t = *(const float2*)&Us[x * 4 * UQ + mb * 16 * HN];
                    af[buf][x][mb][0] = t.x;
                    af[buf][x][mb][1] = t.y;
                }
        }
    };
    auto load_rows = [&](auto setc, int chunk) {
        constexpr int set = decltype(setc)::value;
        const uint32_t c0_bytes = (uint32_t)(chunk * CB) * chan_bytes;
#pragma unroll
        for (int i = 0; i < LBE; ++i)
#pragma unroll
            for (int c = 0; c < CB; ++c)
                r_reg[set][i][c] = __builtin_bit_cast(
                    float, __builtin_amdgcn_raw_buffer_load_b32(rin, (int)r_goff[i], (int)(c0_bytes + (uint32_t)c * chan_bytes), 0));
    };
    auto store_rows = [&](auto setc, auto bufc) {
        constexpr int set = decltype(setc)::value, buf = decltype(bufc)::value;
#pragma unroll
        for (int i = 0; i < LBE; ++i) {
            if (r_lds[i] >= 0) {
                float* dst = Rs0 + buf * CB * raw_chan + r_lds[i];
#pragma unroll
                for (int c = 0; c < CB; ++c) {
                    *dst = r_reg[set][i][c];
                    dst += raw_chan;
                }
            }
        }
    };

    // ---- input transform: thread = (tile, channel of the step) ---------------------------------------------------------
    const bool v_task = tid < TT * CB;
    const int v_c = tid / TT, v_tl = tid % TT;  // tiles along the lanes: LDS reads and writes of a wave are contiguous runs
    int v_src;
    {
        const int t = (t0 + v_tl < geo.tiles) ? t0 + v_tl : t0;  // tiles past the end repeat the first one; never stored
        uint32_t g, tx;
        a.dX.divmod((uint32_t)t, g, tx);
        v_src = v_c * raw_chan + (int)(g - g_first) * 4 * PWL + 2 * (int)tx;
    }
    const int v_dst = v_c * VP + v_tl;

    float2 d_lo[4], d_hi[4];  // the 4x4 input tile between its LDS reads and its use
    auto transform_read = [&](auto bufc) {
        constexpr int buf = decltype(bufc)::value;
        if (v_task) {
            const float* src = Rs0 + buf * CB * raw_chan + v_src;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                d_lo[r] = *(const float2*)&src[r * PWL];
                d_hi[r] = *(const float2*)&src[r * PWL + 2];
            }
        }
    };
    auto transform_write = [&](auto bufc) {
        constexpr int buf = decltype(bufc)::value;
        if (v_task) {
            float d[4][4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                d[r][0] = d_lo[r].x; d[r][1] = d_lo[r].y; d[r][2] = d_hi[r].x; d[r][3] = d_hi[r].y;
            }
            // B^T d B with B^T = [1 0 -1 0; 0 1 1 0; 0 -1 1 0; 0 1 0 -1]
            float t[4][4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                t[0][j] = d[0][j] - d[2][j];
                t[1][j] = d[1][j] + d[2][j];
                t[2][j] = d[2][j] - d[1][j];
                t[3][j] = d[1][j] - d[3][j];
            }
            float* Vs = Vs0 + buf * V_FLOATS + v_dst;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                Vs[(4 * i + 0) * CB * VP] = t[i][0] - t[i][2];
                Vs[(4 * i + 1) * CB * VP] = t[i][1] + t[i][2];
                Vs[(4 * i + 2) * CB * VP] = t[i][2] - t[i][1];
                Vs[(4 * i + 3) * CB * VP] = t[i][1] - t[i][3];
            }
        }
    };

    typename mma_t::acc_t acc[XW][MBLK][NBLK];
#pragma unroll
    for (int x = 0; x < XW; ++x)
#pragma unroll
        for (int mb = 0; mb < MBLK; ++mb)
#pragma unroll
            for (int nb = 0; nb < NBLK; ++nb)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[x][mb][nb][v] = 0.0f;

    // lane (li, kq) feeds column li of a block with channel kq + 4*h in the h-th MFMA of a step
    auto read_tiles = [&](auto bufc) {
        constexpr int buf = decltype(bufc)::value;
        const float* Vs = Vs0 + buf * V_FLOATS + (wave * XW * CB + kq) * VP + li;
#pragma unroll
        for (int x = 0; x < XW; ++x)
#pragma unroll
            for (int nb = 0; nb < NBLK; ++nb)
#pragma unroll
                for (int h = 0; h < HN; ++h) bf[buf][x][nb][h] = Vs[(x * CB + 4 * h) * VP + nb * 16];
    };
    // The step's products as NU units: unit u = (reduction group h, plane x, block mb, block nb), h outermost, so that
    // consecutive MFMAs write different accumulators.
    constexpr int NB1 = XW * MBLK * NBLK, NU = HN * NB1;
    auto mma_range = [&](auto bufc, auto u0c, auto u1c) {
        constexpr int buf = decltype(bufc)::value, U0 = decltype(u0c)::value, U1 = decltype(u1c)::value;
#pragma unroll
        for (int u = U0; u < U1; ++u) {
            const int h = u / NB1, x = (u % NB1) / (MBLK * NBLK), mb = (u % (MBLK * NBLK)) / NBLK, nb = u % NBLK;
            acc[x][mb][nb] = mma_t::run(af[buf][x][mb][h], bf[buf][x][nb][h], acc[x][mb][nb]);
        }
    };
    typedef std::integral_constant<int, 0> c0_t;
    typedef std::integral_constant<int, 1> c1_t;
    typedef std::integral_constant<int, NU / 2> u_a;
    typedef std::integral_constant<int, NU - NU / 4> u_b;
    typedef std::integral_constant<int, NU> u_c;

    // ---- pipeline -----------------------------------------------------------------------------------------------------
    // entering step i: Vs[i&1] holds the transformed tiles of step i and fragment set bf[i&1] was read from it; af[i&1]
    // is in flight or loaded; Rs[(i+1)&1] holds the rows of step i+1; r_reg[(i+1)&1] holds the rows of step i+2.
    load_filters(c0_t{}, 0);
    load_raw(c0_t{}, 0);
    load_raw(c1_t{}, 1);
    load_rows(c0_t{}, 0);
    load_rows(c1_t{}, 1);
    for (int i = tid; i < 2 * CB * raw_chan; i += NT) Rs0[i] = 0.0f;  // border and unused rows stay zero for the whole kernel
    __syncthreads();
    store_rows(c0_t{}, c0_t{});
    store_rows(c1_t{}, c1_t{});
    load_rows(c1_t{}, 2);
    __syncthreads();
    transform_read(c0_t{});
    transform_write(c0_t{});
    transform_filters(c0_t{}, c0_t{});
    __syncthreads();
    read_tiles(c0_t{});
    read_filters(c0_t{});

    // One step, one barrier.  The products of step i surround the LDS traffic that prepares steps i+1 and i+2, and the
    // last quarter of them runs after the barrier, behind the reads of the next step's fragments.
    auto body = [&](auto bufc, int i) {
        constexpr int buf = decltype(bufc)::value;
        typedef std::integral_constant<int, buf ^ 1> other_t;
        const bool nxt = i + 1 < chunks, nxt2 = i + 2 < chunks;
        load_filters(other_t{}, i + 1);
        load_raw(bufc, i + 2);   // FF: register set `buf` was transformed in the previous step
        load_rows(bufc, i + 3);
        if (nxt) transform_read(other_t{});
        __builtin_amdgcn_sched_barrier(0);
        mma_range(bufc, c0_t{}, u_a{});
        __builtin_amdgcn_sched_barrier(0);
        if (nxt) transform_write(other_t{});
        if (nxt) transform_filters(other_t{}, other_t{});
        if (nxt2) store_rows(other_t{}, bufc);
        __builtin_amdgcn_sched_barrier(0);
        mma_range(bufc, u_a{}, u_b{});
        __builtin_amdgcn_sched_barrier(0);  // the products above cover the completion of the LDS writes before the barrier
        __syncthreads();
        if (nxt) read_tiles(other_t{});
        if (nxt) read_filters(other_t{});
        __builtin_amdgcn_sched_barrier(0);
        mma_range(bufc, u_b{}, u_c{});
    };
    int chunk = 0;
    for (; chunk + 1 < chunks; chunk += 2) {
        body(c0_t{}, chunk);
        body(c1_t{}, chunk + 1);
    }
    if (chunk < chunks) body(c0_t{}, chunk);
    __syncthreads();  // every wave is done with the operand buffers before the planes overwrite them

    // ---- epilogue: planes to LDS, inverse transform, bias + activation, 2x2 stores -----------------------------------
    float* const Ms = smem;  // [16][TM][MP]
#pragma unroll
    for (int x = 0; x < XW; ++x)
#pragma unroll
        for (int mb = 0; mb < MBLK; ++mb)
#pragma unroll
            for (int nb = 0; nb < NBLK; ++nb)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    Ms[((wave * XW + x) * TM + mb * 16 + kq * 4 + v) * MP + nb * 16 + li] = acc[x][mb][nb][v];
    __syncthreads();

    const __amdgpu_buffer_rsrc_t rbias = make_rsrc(a.bias, a.bias ? (uint32_t)a.K * 4u : 0u);
    const __amdgpu_buffer_rsrc_t rout = make_rsrc(a.out, a.out_bytes);
    constexpr int NE = (TM * TT + NT - 1) / NT;
#pragma unroll
    for (int j = 0; j < NE; ++j) {
        const int e = j * NT + tid;
        const int kl = e / TT, tl = e % TT;
        const int k = m0 + kl, t = t0 + tl;
        const bool ok = e < TM * TT && k < a.K && t < geo.tiles;
        const float* src = Ms + (ok ? kl * MP + tl : 0);
        float m[4][4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) m[i][jj] = src[(4 * i + jj) * TM * MP];
        // A^T m A with A^T = [1 1 1 0; 0 1 -1 -1]
        float r0[4], r1[4];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            r0[jj] = (m[0][jj] + m[1][jj]) + m[2][jj];
            r1[jj] = (m[1][jj] - m[2][jj]) - m[3][jj];
        }
        float y[2][2];
        y[0][0] = (r0[0] + r0[1]) + r0[2];
        y[0][1] = (r0[1] - r0[2]) - r0[3];
        y[1][0] = (r1[0] + r1[1]) + r1[2];
        y[1][1] = (r1[1] - r1[2]) - r1[3];
        uint32_t n, rem, ty, tx;
        a.dZ.divmod(ok ? (uint32_t)t : 0u, n, rem);
        a.dX.divmod(rem, ty, tx);
        const float b = buffer_load_elem<float>(rbias, ok ? (uint32_t)k * 4u : kOutOfRange);
        const int oy = 2 * (int)ty, ox = 2 * (int)tx;
        const uint32_t base = (uint32_t)(((int)n * a.K + k) * a.OHW + oy * a.OW + ox) * 4u;
#pragma unroll
        for (int dy = 0; dy < 2; ++dy)
#pragma unroll
            for (int dx = 0; dx < 2; ++dx) {
                float v = y[dy][dx] + b;
                if (a.relu) v = v > 0.0f ? v : 0.0f;
                const bool in_img = ok && oy + dy < a.OH && ox + dx < a.OW;
                buffer_store_elem<float>(v, rout, in_img ? base + (uint32_t)(dy * a.OW + dx) * 4u : kOutOfRange);
            }
    }
}

template <class CFG>
size_t wino_ws_bytes(const Variant& v, const conv_desc& d, int OH, int OW)
{
    if (CFG::FF || (d.flags & CONV_FLAG_FILT_WINOGRAD)) return 0;  // transformed in the kernel, or handed over by the caller
    return (size_t)16 * wino_kpitch(d.K) * d.C * sizeof(float);
}

template <class CFG>
hipError_t wino_launch(const Variant& v, ConvArgs& a, hipStream_t s)
{
    const size_t lds = wino_lds_bytes<CFG>(a.N, a.OH, a.OW);
    const hipError_t e = ensure_dynamic_lds((const void*)wino_kernel<CFG>, lds);
    if (e != hipSuccess) return e;
    const WinoGeom g = wino_geom<CFG>(a.N, a.OH, a.OW);
    a.nsplit = 1;
    a.steps_per_split = 0;
    a.dX = make_fastdiv((uint32_t)g.TW);
    a.dY = make_fastdiv((uint32_t)g.TH);
    a.dZ = make_fastdiv((uint32_t)g.tiles_img);
    if (CFG::FF) {
        // nothing to prepare: the product kernel reads the filters as they are
    } else if (a.filt_wino) {
        a.ws = (float*)const_cast<void*>(a.filt);  // already in the Winograd domain
    } else {
        hipLaunchKernelGGL(wino_filter_kernel<CFG::CB>, dim3((unsigned)((a.K + 31) / 32), (unsigned)(a.C / CFG::CB)), dim3(32 * CFG::CB), 0, s,
                           (const float*)a.filt, a.ws, a.K, a.C);
        const hipError_t e2 = hipGetLastError();
        if (e2 != hipSuccess) return e2;
    }
    dim3 grid((unsigned)(((g.tiles + CFG::TT - 1) / CFG::TT) * ((a.K + CFG::TM - 1) / CFG::TM)));
    hipLaunchKernelGGL(wino_kernel<CFG>, grid, dim3(CFG::NT), lds, s, a);
    return hipGetLastError();
}

template <class CFG>
bool wino_valid(const Variant& v, const conv_desc& d, int OH, int OW)
{
    if (d.dtype != CONV_F32 || d.R != 3 || d.S != 3 || d.stride != 1 || d.pad > 1) return false;
    if ((d.C % CFG::CB) != 0) return false;
    if ((d.flags & CONV_FLAG_FILT_WINOGRAD) && (CFG::CB != 8 || CFG::FF)) return false;  // the hand-over layout is that of the 8-channel step
    const WinoGeom g = wino_geom<CFG>(d.N, OH, OW);
    // every (input row of the workgroup's tile rows, x) needs a staging slot
    if ((long long)g.nr_max * 4 * d.W > (long long)CFG::NT * CFG::LBE) return false;
    if (wino_lds_bytes<CFG>(d.N, OH, OW) > 160 * 1024) return false;
    // offsets are formed in 32 bits next to an out-of-range marker: input and transformed filters below 2 GiB
    if ((long long)d.N * (d.C + 3 * CFG::CB) * d.H * d.W * 4 >= (1LL << 31)) return false;  // the pipeline looks three steps ahead
    if ((long long)wino_kpitch(d.K) * d.C * 64 >= (1LL << 31)) return false;
    if (d.C / CFG::CB > 65535) return false;
    if ((long long)d.N * g.tiles_img >= (1LL << 30)) return false;
    if ((long long)((d.K + CFG::TM - 1) / CFG::TM) * ((g.tiles + CFG::TT - 1) / CFG::TT) >= (1LL << 31)) return false;
    return true;
}

template <class CFG>
void wino_register(std::vector<Variant>& out)
{
    Variant v;
    char buf[96];
    snprintf(buf, sizeof buf, "wino_f32_M%dT%d_x%d_c%d_e%d%s", CFG::TM, CFG::TT, CFG::XW, CFG::CB, CFG::LBE, CFG::FF ? "_ff" : "");
    v.name = buf;
    v.dtype = CONV_F32;
    v.split = 1;
    v.tm = CFG::TM;
    v.tn = CFG::TT * 4;
    v.tk = CFG::CB * 9;
    v.threads = CFG::NT;
    v.family = FAM_WINOGRAD;
    v.specificity = 5;
    v.valid = &wino_valid<CFG>;
    v.launch = &wino_launch<CFG>;
    v.ws_extra = &wino_ws_bytes<CFG>;
    if (CFG::FF) v.traits |= TRAIT_FILTERS_IN_KERNEL;
    out.push_back(v);
}

}  // namespace convfwd
