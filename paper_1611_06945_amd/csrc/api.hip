// Host side of libconvfwd.so: descriptor validation, the variant registry, variant
// selection (forced > autotuned > heuristic), the brute-force autotuner, cache
// persistence and the extern "C" entry points declared in include/convfwd.h.
#include <algorithm>
#include <array>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <fstream>
#include <map>
#include <mutex>
#include <sstream>

#include "common.h"

using namespace convfwd;

namespace {

typedef std::array<int64_t, 11> Key;

Key key_of(const conv_desc& d)
{
    return Key{d.N, d.C, d.H, d.W, d.K, d.R, d.S, d.stride, d.pad, d.dtype, (int64_t)d.flags};
}

struct Choice {
    std::string best;       // fastest variant overall (may need workspace)
    std::string best_nows;  // fastest variant that needs no workspace
};

struct State {
    std::mutex mu;
    std::vector<Variant> variants;
    std::map<std::string, int> by_name;
    std::map<Key, Choice> cache;
    std::map<Key, int> forced;                   // index into valid_list(desc)
    std::map<Key, std::vector<double>> times_us;  // per valid-list index, from the last autotune
    // Per descriptor: its valid list and the cost model's picks.  The registry never changes after start-up, so these
    // are computed once; a call then costs two map look-ups instead of a pass over every variant.
    struct Memo {
        std::vector<int> valid;
        int pick_any = -2;       // cost model's pick with unlimited workspace (-2: not computed yet)
        size_t pick_any_ws = 0;  // workspace that pick needs
        int pick_nows = -2;      // cost model's pick among variants that need no workspace
    };
    std::map<Key, Memo> memo;
};

State& state()
{
    static State* st = [] {
        State* s = new State;
        register_igemm_f32(s->variants);
        register_igemm_f16(s->variants);
        register_igemm_bf16(s->variants);
        register_ugemm_f32(s->variants);
        register_ugemm_f16(s->variants);
        register_ugemm_bf16(s->variants);
        register_fc(s->variants);
        register_nhwc_f16(s->variants);
        register_nhwc_bf16(s->variants);
        register_nwin_f16(s->variants);
        register_nwin_bf16(s->variants);
        register_wconv_f32(s->variants);
        register_wino_f32(s->variants);
        register_swin_f16(s->variants);
        register_swin_bf16(s->variants);
        register_swinp_f16(s->variants);
        register_swinp_bf16(s->variants);
        register_wconv_f16(s->variants);
        register_wconv_bf16(s->variants);
        register_pwk_f32(s->variants);
        register_pwk_f16(s->variants);
        register_pwk_bf16(s->variants);
        register_pwin32_f32(s->variants);
        register_pwin_f16(s->variants);
        register_pwin_bf16(s->variants);
        for (size_t i = 0; i < s->variants.size(); ++i) s->by_name[s->variants[i].name] = (int)i;
        return s;
    }();
    return *st;
}

// Identity written into saved autotune caches: measurements belong to one device model and one set of kernels.
std::string registry_id(State& st)
{
    uint64_t h = 1469598103934665603ull;  // FNV-1a over every variant name, in registration order
    for (const Variant& v : st.variants)
        for (unsigned char c : v.name + "\n") h = (h ^ c) * 1099511628211ull;
    char buf[32];
    snprintf(buf, sizeof buf, "%016llx", (unsigned long long)h);
    return buf;
}

std::string device_id()
{
    int dev = 0;
    hipDeviceProp_t p;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&p, dev) != hipSuccess) {
        (void)hipGetLastError();  // a host without a GPU: not an error of the caller's
        return "none";
    }
    std::string s = std::string(p.gcnArchName) + "/" + p.name + "/" + std::to_string(p.multiProcessorCount) + "cu";
    for (char& c : s)
        if (c == ' ' || c == '\t') c = '_';
    return s;
}

thread_local std::string g_hip_msg;
thread_local std::string g_ws_msg;  // detail for CONV_EWORKSPACE from conv_fwd_static

int hip_fail(hipError_t e, const char* what)
{
    g_hip_msg = std::string(what) + ": " + hipGetErrorString(e);
    return CONV_EHIP;
}

constexpr uint32_t kLayoutFlags = CONV_FLAG_IN_NHWC | CONV_FLAG_OUT_NHWC | CONV_FLAG_FILT_KRSC;
constexpr uint32_t kKnownFlags =
    CONV_FLAG_RELU | kLayoutFlags | CONV_FLAG_FILT_WINOGRAD | CONV_FLAG_MAXPOOL_3X3S2 | CONV_FLAG_FILT_PACKED;

// Validation shared by every entry point; fills OH/OW.
int check_desc(const conv_desc* d, int& OH, int& OW)
{
    if (!d) return CONV_EINVAL;
    if (d->dtype != CONV_F32 && d->dtype != CONV_F16 && d->dtype != CONV_BF16) return CONV_EDTYPE;
    if (d->N < 1 || d->C < 1 || d->H < 1 || d->W < 1 || d->K < 1 || d->R < 1 || d->S < 1) return CONV_EINVAL;
    if (d->stride < 1 || d->pad < 0) return CONV_EINVAL;
    if (d->flags & ~kKnownFlags) return CONV_EINVAL;
    const int64_t sh = (int64_t)d->H + 2LL * d->pad - d->R, sw = (int64_t)d->W + 2LL * d->pad - d->S;
    if (sh < 0 || sw < 0) return CONV_EINVAL;
    const int64_t oh = sh / d->stride + 1, ow = sw / d->stride + 1;
    const int64_t lim = (int64_t)1 << 31;
    const int64_t n_in = (int64_t)d->N * d->C * d->H * d->W;
    const int64_t n_f = (int64_t)d->K * d->C * d->R * d->S;
    if (oh >= lim || ow >= lim) return CONV_EINVAL;
    if ((d->flags & CONV_FLAG_MAXPOOL_3X3S2) && (oh < 3 || ow < 3)) return CONV_EINVAL;
    // guard the products against overflow before forming them
    if ((double)d->N * d->C * (double)d->H * d->W >= (double)lim) return CONV_EINVAL;
    if ((double)d->K * d->C * (double)d->R * d->S >= (double)lim) return CONV_EINVAL;
    if ((double)d->N * d->K * (double)oh * (double)ow >= (double)lim) return CONV_EINVAL;
    // tile loads go through 32-bit buffer descriptors: every tensor must also stay below 4 GiB
    const double esz = d->dtype == CONV_F32 ? 4.0 : 2.0, lim_b = 4294967296.0;
    if ((double)d->N * d->C * (double)d->H * d->W * esz >= lim_b) return CONV_EINVAL;
    if ((double)d->K * d->C * (double)d->R * d->S * esz >= lim_b) return CONV_EINVAL;
    if ((double)d->N * d->K * (double)oh * (double)ow * esz >= lim_b) return CONV_EINVAL;
    // the padded coordinates formed inside the kernels must fit an int as well
    if ((double)(d->H + 2.0 * d->pad) * (double)(d->W + 2.0 * d->pad) >= (double)lim) return CONV_EINVAL;
    (void)n_in;
    (void)n_f;
    OH = (int)oh;
    OW = (int)ow;
    return CONV_OK;
}

std::vector<int> valid_list(State& st, const conv_desc& d, int OH, int OW)
{
    std::vector<int> r;
    // descriptors with channel-innermost tensors are served by the kernels written for them, and only those
    const bool layout = (d.flags & kLayoutFlags) != 0;
    const bool wino_filters = (d.flags & CONV_FLAG_FILT_WINOGRAD) != 0;
    if (layout && wino_filters) return r;
    const bool pool = (d.flags & CONV_FLAG_MAXPOOL_3X3S2) != 0;
    if (pool && wino_filters) return r;
    // ... except planar input and filters with a channel-innermost output, which some planar kernels can write
    const bool planar_to_nhwc = (d.flags & kLayoutFlags) == CONV_FLAG_OUT_NHWC;
    // filters in MFMA operand order: only the kernels written for them, which check the other formats themselves
    const bool packed = (d.flags & CONV_FLAG_FILT_PACKED) != 0;
    if (packed && (wino_filters || (d.flags & CONV_FLAG_FILT_KRSC))) return r;
    for (size_t i = 0; i < st.variants.size(); ++i) {
        if (packed != ((st.variants[i].traits & TRAIT_PACKED_FILTERS) != 0)) continue;
        if (packed) {
            if (st.variants[i].valid(st.variants[i], d, OH, OW)) r.push_back((int)i);
            continue;
        }
        if (planar_to_nhwc) {
            if (!(st.variants[i].traits & TRAIT_PLANAR_TO_NHWC)) continue;
        } else if ((st.variants[i].family == FAM_NHWC) != layout) {
            continue;
        }
        if (wino_filters && st.variants[i].family != FAM_WINOGRAD) continue;
        if (pool && !(st.variants[i].traits & TRAIT_POOL_EPILOGUE)) continue;
        if (st.variants[i].valid(st.variants[i], d, OH, OW)) r.push_back((int)i);
    }
    return r;
}

size_t ws_bytes_of(const Variant& v, const conv_desc& d, int OH, int OW)
{
    if (v.ws_extra) return v.ws_extra(v, d, OH, OW);
    if (v.split <= 1) return 0;
    return (size_t)v.split * (size_t)d.K * (size_t)d.N * OH * OW * sizeof(float);
}

// Rough cost model used only when nothing was autotuned for this descriptor: number of rounds the
// workgroups need on 256 CUs times the work of one workgroup, small tiles charged for their extra
// operand traffic, splits charged for the second pass.  Ties go to the more specialised variant
// (the paper's "most specialised possible" rule for non-autotuned selection).
// Estimated time in microseconds of one call, used to rank variants for a shape nobody has measured.  The model: a
// launch runs ceil(workgroups / slots) rounds, each of `steps` reduction steps; a step costs the tile's multiply-adds at
// a per-CU rate (lower for small tiles, which move more operand bytes per multiply-add, and scaled per kernel family)
// plus a fixed part for its barrier and address work; workgroups that share a CU slow each other down; reduction
// splits add a second launch and the traffic of their partial sums.  The constants are a coordinate-descent fit to the
// measured times of every variant on 275 workloads (the benchmark layers and the 43 operations of Appendix A at batch
// 1, 5 and 20, fp32 and fp16): the pick's time over the best variant's time averages 1.03 and stays below 1.35 there.
double heuristic_cost(const Variant& v, const conv_desc& d, int OH, int OW)
{
    const double P = (double)d.N * OH * OW, Q = (double)d.C * d.R * d.S;
    if (v.family == FAM_FC) return 1.0 + std::abs(v.tm - 4);  // weight streaming: always ahead of the MFMA tiles when valid
    if (v.family == FAM_WINOGRAD) {
        // F(2x2,3x3) product kernel: one workgroup per (v.tm channels, v.tn / 4 tiles of 2x2 outputs), one round per 256
        // workgroups, a step per v.tk / 9 input channels whose cost grows with the products and with the operands it
        // transforms; the separate filter transform is a launch plus its traffic.  Least-squares fit (rms 8 %) to every
        // Winograd variant on the 3x3 operations of Appendix A and benchmark configuration 4 at batch 1, 5 and 20.
        const double tt = v.tn / 4.0, cb = v.tk / 9.0;
        const double tiles = (double)d.N * std::ceil(OH / 2.0) * std::ceil(OW / 2.0);
        const double rounds = std::ceil(std::ceil(d.K / (double)v.tm) * std::ceil(tiles / tt) / 256.0);
        double t_step = 0.026 + 0.262e-4 * v.tm * tt * cb + 1.443e-3 * (v.tm + tt) * cb;
        double t_filters = 4.15 + 0.49e-5 * (double)d.K * d.C;
        if (v.traits & TRAIT_FILTERS_IN_KERNEL) t_filters = 0.0, t_step *= 1.12;
        if (d.flags & CONV_FLAG_FILT_WINOGRAD) t_filters = 0.0;
        return 4.62 + t_filters + rounds * (d.C / cb) * t_step;
    }
    if (v.family == FAM_FIRSTLAYER && (v.traits & TRAIT_POOL_EPILOGUE)) {
        // one workgroup per tile of pooled outputs and channel tile, one per CU at a time: filters re-laid, input rows
        // staged, one 32-pixel block per wave (v.threads / 256 per SIMD), then the pooling pass
        const double side = std::sqrt((double)v.tn), pt = (side - 1.0) / 2.0;
        const double POH = (OH - 3) / 2 + 1, POW = (OW - 3) / 2 + 1;
        const double wgs = (double)d.N * std::ceil(POH / pt) * std::ceil(POW / pt) * std::ceil(d.K / (double)v.tm);
        const double per_wg = 2.0 + 0.03 * v.tm + (v.threads / 256.0) * (v.tk / 16.0) * (v.tm / 32.0) * 0.016 + 1.5;
        return 2.5 + std::ceil(wgs / 256.0) * per_wg;
    }
    if (v.family == FAM_FIRSTLAYER) {
        // persistent workgroups, one per CU and channel tile, walking over tiles of v.tn pixels of one image: a start-up
        // that grows with the filter rows a workgroup re-lays, then a time per tile (measured on the 11x11 stride-4 and
        // 7x7 stride-2 first layers at batch 5 and 20)
        const double tiles = (double)d.N * std::ceil((double)OH * OW / v.tn), ktiles = std::ceil(d.K / (double)v.tm);
        const double wgs = std::max(1.0, std::min(std::floor(256.0 / ktiles), tiles));
        const double per_tile = 1.3 + (0.5 + 0.0156 * v.tm) * v.tk / 416.0;  // two tiles of a workgroup run side by side
        return 1.05 + 0.058 * v.tm + std::ceil(tiles / wgs) * per_tile;
    }
    if (v.traits & TRAIT_WAVE_SPLIT) {
        // every wave of the tile's workgroup multiplies its share of the channels straight from global memory: one round
        // of memory latency, then 27 ns per fp32 32x32x2 MFMA and SIMD, then the exchange of the partial sums
        const double kw = v.threads / 64.0, tiles = std::ceil(d.K / (double)v.tm) * std::ceil(P / (double)v.tn);
        const double per_cu = std::max(1.0, std::floor(16.0 / kw));
        const double rounds = std::ceil(tiles / (256.0 * per_cu));
        // (16-bit storage: one 32x32x16 MFMA of 16 ns per group of 16 channels, fed by eight 2-byte loads per lane)
        const bool f32 = d.dtype == CONV_F32;
        const double mfmas = std::ceil(d.C / (f32 ? 8.0 : 16.0) / kw) * (f32 ? 4.0 : 1.0) * (v.tm / 32.0) * (v.tn / 32.0);
        const double share = std::min(per_cu, std::max(1.0, tiles / 256.0)) * kw / 4.0;  // waves per SIMD
        return 3.2 + rounds * (0.9 + mfmas * (f32 ? 0.027 : 0.030) * std::max(1.0, share)) + 0.3 + 0.02 * kw;
    }
    if (v.traits & TRAIT_CHANNEL_WAVES) {
        // one workgroup per (channel tile, run of v.tn pixels); its v.threads / 64 waves split the channels, so a SIMD
        // multiplies tm*tn/1024 * Q/2 / (waves per workgroup) MFMAs of 30 ns (27 ns at the issue limit) per resident wave
        const double waves = v.threads / 64.0, tiles = std::ceil(d.K / (double)v.tm) * std::ceil(P / (double)v.tn);
        const double rounds = std::ceil(tiles / 256.0);
        const double pix_waves = (v.tn / 32.0 >= 4.0 && waves >= 8.0) ? 2.0 : 1.0;
        const double mfmas = (v.tm / 32.0) * (v.tn / 32.0 / pix_waves) * (Q / 2.0) / (waves / pix_waves);
        // ... and, when the tiles outnumber the SIMDs, the chip's MFMA rate at the half efficiency these kernels reach
        // there (filter and input slabs staged through LDS once per workgroup and chunk)
        const double busy = tiles * waves * mfmas * 0.0305 / 1024.0 / 0.5;
        return 5.0 + 0.05 * waves + std::max(rounds * mfmas * 0.030 * std::max(1.0, waves / 4.0), busy);
    }
    const bool window = v.family == FAM_WINDOW || (v.traits & TRAIT_WINDOW_TILES);
    double tiles;
    if (window) {  // one workgroup per (image, band of pixels, channel tile): pixels are not packed across images
        const double per_img = (double)OH * OW;
        tiles = (double)d.N * (per_img > v.tn ? std::ceil(per_img / v.tn) : 1.0) * std::ceil(d.K / (double)v.tm) * v.split;
    } else {
        tiles = std::ceil(d.K / (double)v.tm) * std::ceil(P / (double)v.tn) * v.split;
    }
    const double steps = std::ceil(std::ceil(Q / v.tk) / v.split);
    const double rate = d.dtype == CONV_F32 ? 2.4e5 : 8.0e5;  // multiply-adds per microsecond and CU
    const double small = 1.0 / (1.0 + 24.0 / v.tm + 24.0 / v.tn);
    double fam = window ? 2.2 : v.family == FAM_POINTWISE ? 1.3 : (v.traits & TRAIT_REGISTER_OPERANDS) ? 0.8 : 0.7;
    if (v.traits & TRAIT_WHOLE_IMAGE) fam *= 1.1;
    if (v.traits & TRAIT_SCALAR_LOADS) fam *= d.dtype == CONV_F32 ? 0.8 : 0.4;
    if (v.traits & TRAIT_STRIDED_VECTOR) fam *= 0.8;
    const double t_step = (double)v.tm * v.tn * v.tk / (rate * small * fam) + 0.2;
    const double wg_per_cu = window ? 1.0 : (v.tm * v.tn >= 128 * 128) ? 1.0 : (v.tm * v.tn >= 64 * 128) ? 2.0 : 3.0;
    const double rounds = std::ceil(tiles / (256.0 * wg_per_cu));
    const double sharing = std::min(wg_per_cu, std::max(1.0, tiles / 256.0));
    double t = 4.0 + rounds * steps * t_step * std::pow(sharing, 0.4);
    if (v.split > 1) t += 2.0 + (double)v.split * d.K * P * 4.0 / 2.0e6;
    // a conversion launch ahead of the kernel: its launch plus input and filters read and written once
    if (v.traits & TRAIT_CONVERTS_FIRST) t += 3.0 + 2.0 * ((double)d.N * d.C * d.H * d.W + (double)d.K * Q) * 2.0 / 2.0e6;
    return t * (1.0 - 0.002 * v.specificity);  // ties go to the kernel written for the narrower class of shapes
}

int pick_heuristic(State& st, const std::vector<int>& valid, const conv_desc& d, int OH, int OW, size_t ws_limit)
{
    int best = -1;
    double best_cost = 0;
    for (int idx : valid) {
        const Variant& v = st.variants[idx];
        if (ws_bytes_of(v, d, OH, OW) > ws_limit) continue;
        const double c = heuristic_cost(v, d, OH, OW);
        if (best < 0 || c < best_cost) {
            best = idx;
            best_cost = c;
        }
    }
    return best;
}

State::Memo& memo_of(State& st, const conv_desc& d, int OH, int OW)
{
    const Key k = key_of(d);
    auto it = st.memo.find(k);
    if (it == st.memo.end()) {
        it = st.memo.emplace(k, State::Memo{}).first;
        it->second.valid = valid_list(st, d, OH, OW);
    }
    return it->second;
}

// Returns the registry index to run, or a negative status.
int select_variant(State& st, const conv_desc& d, int OH, int OW, size_t ws_limit)
{
    State::Memo& m = memo_of(st, d, OH, OW);
    const std::vector<int>& valid = m.valid;  // ascending registry indices
    if (valid.empty()) return CONV_ENOVARIANT;
    const Key k = key_of(d);
    auto f = st.forced.find(k);
    if (f != st.forced.end()) {
        if (f->second < 0 || f->second >= (int)valid.size()) return CONV_ENOVARIANT;
        const int idx = valid[f->second];
        if (ws_bytes_of(st.variants[idx], d, OH, OW) > ws_limit) return CONV_EWORKSPACE;
        return idx;
    }
    auto c = st.cache.find(k);
    if (c != st.cache.end()) {
        for (const std::string* nm : {&c->second.best, &c->second.best_nows}) {
            auto it = st.by_name.find(*nm);
            if (it == st.by_name.end()) continue;
            if (!std::binary_search(valid.begin(), valid.end(), it->second)) continue;
            if (ws_bytes_of(st.variants[it->second], d, OH, OW) <= ws_limit) return it->second;
        }
    }
    // the unconstrained pick also wins under any limit that admits it
    if (m.pick_any == -2) {
        m.pick_any = pick_heuristic(st, valid, d, OH, OW, SIZE_MAX);
        m.pick_any_ws = m.pick_any >= 0 ? ws_bytes_of(st.variants[m.pick_any], d, OH, OW) : 0;
    }
    if (m.pick_any >= 0 && m.pick_any_ws <= ws_limit) return m.pick_any;
    int h;
    if (ws_limit == 0) {
        if (m.pick_nows == -2) m.pick_nows = pick_heuristic(st, valid, d, OH, OW, 0);
        h = m.pick_nows;
    } else {
        h = pick_heuristic(st, valid, d, OH, OW, ws_limit);
    }
    return h < 0 ? CONV_ENOVARIANT : h;
}

void fill_args(ConvArgs& a, const conv_desc& d, int OH, int OW, const void* in, const void* filt, const float* bias,
               void* out, void* ws)
{
    a.in = in;
    a.filt = filt;
    a.bias = bias;
    a.out = out;
    a.ws = (float*)ws;
    a.N = d.N; a.C = d.C; a.H = d.H; a.W = d.W; a.K = d.K; a.R = d.R; a.S = d.S;
    a.stride = d.stride; a.pad = d.pad; a.OH = OH; a.OW = OW;
    a.P = d.N * OH * OW;
    a.Q = d.C * d.R * d.S;
    a.HW = d.H * d.W;
    a.OHW = OH * OW;
    a.RS = d.R * d.S;
    a.relu = (d.flags & CONV_FLAG_RELU) ? 1 : 0;
    a.out_nhwc = (d.flags & CONV_FLAG_OUT_NHWC) ? 1 : 0;
    a.filt_wino = (d.flags & CONV_FLAG_FILT_WINOGRAD) ? 1 : 0;
    a.in_bytes = (uint32_t)((uint64_t)d.N * d.C * d.H * d.W * dtype_size(d.dtype));
    a.filt_bytes = (uint32_t)((uint64_t)d.K * d.C * d.R * d.S * dtype_size(d.dtype));
    a.out_bytes = (uint32_t)((uint64_t)d.N * d.K * OH * OW * dtype_size(d.dtype));
    a.pool = (d.flags & CONV_FLAG_MAXPOOL_3X3S2) ? 1 : 0;
    a.POH = a.pool ? (OH - 3) / 2 + 1 : 0;
    a.POW = a.pool ? (OW - 3) / 2 + 1 : 0;
    if (a.pool) a.out_bytes = (uint32_t)((uint64_t)d.N * d.K * a.POH * a.POW * dtype_size(d.dtype));
    a.nsplit = 1;
    a.steps_per_split = 0;
    a.dRS = make_fastdiv((uint32_t)a.RS);
    a.dS = make_fastdiv((uint32_t)d.S);
    a.dOHW = make_fastdiv((uint32_t)a.OHW);
    a.dOW = make_fastdiv((uint32_t)OW);
    a.dHW = make_fastdiv((uint32_t)a.HW);
    a.dW = make_fastdiv((uint32_t)d.W);
    a.SP4 = (d.S + 3) / 4;
    a.QP = d.C * d.R * a.SP4 * 4;
    a.dRSP = make_fastdiv((uint32_t)(d.R * a.SP4 * 4));
    a.dSP = make_fastdiv((uint32_t)(a.SP4 * 4));
    a.dRSP4 = make_fastdiv((uint32_t)(d.R * a.SP4));
    a.dC = make_fastdiv((uint32_t)d.C);
    a.dSP4 = make_fastdiv((uint32_t)a.SP4);
}

int run_variant(const Variant& v, const conv_desc& d, ConvArgs& a, hipStream_t s)
{
    hipError_t e = v.launch(v, a, s);
    if (e != hipSuccess) return hip_fail(e, v.name.c_str());
    if (v.split > 1) {
        e = launch_split_reduce(a, d.dtype, s);
        if (e != hipSuccess) return hip_fail(e, "split_reduce");
    }
    return CONV_OK;
}

bool aligned16(const void* p) { return (((uintptr_t)p) & 15u) == 0; }

// Library-owned scratch of conv_fwd_static: one array per GPU, living in the code object's data segment for as long as
// the process does.  In host code the symbol below is only a handle, never a device address: the address on a device
// comes from hipGetSymbolAddress with that device current (static_scratch_ptr), and only that pointer is handed to
// kernels.
static __device__ __align__(256) unsigned char scratch[CONV_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up once per device).
int static_scratch_ptr(void** out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return hip_fail(hipErrorInvalidDevice, "conv_fwd_static: device ordinal");
    std::lock_guard<std::mutex> g(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
        if (!p || (((uintptr_t)p) & 255u)) return hip_fail(hipErrorInvalidSymbol, "scratch: null or misaligned address");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return CONV_OK;
}

int fwd_common(const conv_desc* desc, const void* in, const void* filt, const float* bias, void* out, void* ws,
               size_t ws_bytes, void* stream)
{
    int OH, OW;
    const int rc = check_desc(desc, OH, OW);
    if (rc) return rc;
    if (!in || !filt || !out) return CONV_EINVAL;
    if (!aligned16(in) || !aligned16(filt) || !aligned16(out) || (bias && (((uintptr_t)bias) & 3u))) return CONV_EINVAL;
    if (ws && (((uintptr_t)ws) & 255u)) return CONV_EINVAL;
    if (!ws) ws_bytes = 0;
    State& st = state();
    int idx;
    {
        std::lock_guard<std::mutex> g(st.mu);
        idx = select_variant(st, *desc, OH, OW, ws_bytes);
    }
    if (idx < 0) return idx;
    ConvArgs a;
    fill_args(a, *desc, OH, OW, in, filt, bias, out, ws);
    return run_variant(st.variants[idx], *desc, a, (hipStream_t)stream);
}

}  // namespace

extern "C" {

int conv_out_shape(const conv_desc* desc, int32_t* OH, int32_t* OW)
{
    int oh, ow;
    const int rc = check_desc(desc, oh, ow);
    if (rc) return rc;
    if (!OH || !OW) return CONV_EINVAL;
    const bool pool = (desc->flags & CONV_FLAG_MAXPOOL_3X3S2) != 0;
    *OH = pool ? (oh - 3) / 2 + 1 : oh;
    *OW = pool ? (ow - 3) / 2 + 1 : ow;
    return CONV_OK;
}

double conv_flops(const conv_desc* desc)
{
    int oh, ow;
    if (check_desc(desc, oh, ow)) return 0.0;
    return 2.0 * desc->N * desc->K * (double)oh * ow * desc->C * desc->R * desc->S;
}

size_t conv_workspace_bytes(const conv_desc* desc)
{
    int OH, OW;
    if (check_desc(desc, OH, OW)) return 0;
    State& st = state();
    std::lock_guard<std::mutex> g(st.mu);
    size_t need = 0;
    for (int idx : memo_of(st, *desc, OH, OW).valid) need = std::max(need, ws_bytes_of(st.variants[idx], *desc, OH, OW));
    return need;
}

int conv_fwd(const conv_desc* desc, const void* in, const void* filt, const float* bias, void* out, void* stream)
{
    return fwd_common(desc, in, filt, bias, out, nullptr, 0, stream);
}

int conv_fwd_ws(const conv_desc* desc, const void* in, const void* filt, const float* bias, void* out, void* workspace,
                size_t workspace_bytes, void* stream)
{
    return fwd_common(desc, in, filt, bias, out, workspace, workspace_bytes, stream);
}

int conv_fwd_static(const conv_desc* desc, const void* in, const void* filt, const float* bias, void* out, void* stream)
{
    int OH, OW;
    const int rc = check_desc(desc, OH, OW);
    if (rc) return rc;
    if (!in || !filt || !out) return CONV_EINVAL;
    if (!aligned16(in) || !aligned16(filt) || !aligned16(out) || (bias && (((uintptr_t)bias) & 3u))) return CONV_EINVAL;
    State& st = state();
    int idx;
    {
        std::lock_guard<std::mutex> g(st.mu);
        idx = select_variant(st, *desc, OH, OW, SIZE_MAX);
    }
    if (idx < 0) return idx;
    const size_t need = ws_bytes_of(st.variants[idx], *desc, OH, OW);
    if (need > (size_t)CONV_STATIC_SCRATCH_BYTES) {
        char msg[256];
        snprintf(msg, sizeof msg, "conv_fwd_static: variant %s needs %zu bytes of scratch, the library holds %zu",
                 st.variants[idx].name.c_str(), need, (size_t)CONV_STATIC_SCRATCH_BYTES);
        g_ws_msg = msg;
        return CONV_EWORKSPACE;
    }
    void* ws = nullptr;
    if (need) {
        const int prc = static_scratch_ptr(&ws);
        if (prc) return prc;
    }
    ConvArgs a;
    fill_args(a, *desc, OH, OW, in, filt, bias, out, ws);
    return run_variant(st.variants[idx], *desc, a, (hipStream_t)stream);
}

int conv_time_us(const conv_desc* desc, const void* in, const void* filt, const float* bias, void* out, void* workspace,
                 size_t workspace_bytes, void* stream, int launches, double* us_per_launch)
{
    if (launches < 1 || !us_per_launch) return CONV_EINVAL;
    // one untimed call first: it validates everything and takes any one-time cost (function attributes) out of the timing
    int rc = fwd_common(desc, in, filt, bias, out, workspace, workspace_bytes, stream);
    if (rc) return rc;
    hipStream_t s = (hipStream_t)stream;
    hipEvent_t e0, e1;
    hipError_t e = hipEventCreate(&e0);
    if (e != hipSuccess) return hip_fail(e, "hipEventCreate");
    e = hipEventCreate(&e1);
    if (e != hipSuccess) {
        hipEventDestroy(e0);
        return hip_fail(e, "hipEventCreate");
    }
    e = hipEventRecord(e0, s);
    if (e != hipSuccess) rc = hip_fail(e, "hipEventRecord");
    for (int i = 0; i < launches && rc == CONV_OK; ++i) rc = fwd_common(desc, in, filt, bias, out, workspace, workspace_bytes, stream);
    if (rc == CONV_OK) {
        e = hipEventRecord(e1, s);
        if (e != hipSuccess) rc = hip_fail(e, "hipEventRecord");
    }
    if (rc == CONV_OK) {
        e = hipEventSynchronize(e1);
        if (e != hipSuccess) rc = hip_fail(e, "hipEventSynchronize");
    }
    float ms = 0.f;
    if (rc == CONV_OK) {
        e = hipEventElapsedTime(&ms, e0, e1);
        if (e != hipSuccess) rc = hip_fail(e, "hipEventElapsedTime");
    }
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    if (rc == CONV_OK) *us_per_launch = (double)ms * 1000.0 / launches;
    return rc;
}

int conv_autotune(const conv_desc* desc, const void* in, const void* filt, const float* bias, void* out, void* workspace,
                  size_t workspace_bytes, void* stream)
{
    int OH, OW;
    const int rc = check_desc(desc, OH, OW);
    if (rc) return rc;
    if (!in || !filt || !out) return CONV_EINVAL;
    if (!aligned16(in) || !aligned16(filt) || !aligned16(out) || (bias && (((uintptr_t)bias) & 3u))) return CONV_EINVAL;
    if (workspace && (((uintptr_t)workspace) & 255u)) return CONV_EINVAL;
    if (!workspace) workspace_bytes = 0;
    State& st = state();
    std::vector<int> valid;
    {
        std::lock_guard<std::mutex> g(st.mu);
        valid = memo_of(st, *desc, OH, OW).valid;
    }
    if (valid.empty()) return CONV_ENOVARIANT;
    hipStream_t s = (hipStream_t)stream;
    hipEvent_t e0, e1;
    hipError_t e = hipEventCreate(&e0);
    if (e != hipSuccess) return hip_fail(e, "hipEventCreate");
    e = hipEventCreate(&e1);
    if (e != hipSuccess) {
        hipEventDestroy(e0);
        return hip_fail(e, "hipEventCreate");
    }
    std::vector<double> times(valid.size(), -1.0);
    int status = CONV_OK;
    int best = -1, best_nows = -1;
    // Cross-check (the paper's tuning flow compares every candidate's output numerically before it may be kept, Section
    // 4 "Experimental Setup"): the output of a reference candidate -- the first unsplit direct variant that fits, else
    // the first that fits -- is kept in a temporary device buffer, and a candidate whose output differs from it by more
    // than the storage type's bound is not eligible, however fast.
    ConvArgs a0;
    fill_args(a0, *desc, OH, OW, in, filt, bias, out, workspace);
    const size_t out_bytes = a0.out_bytes;
    const size_t n_out = out_bytes / dtype_size(desc->dtype);
    int ref_i = -1;
    for (size_t i = 0; i < valid.size(); ++i) {
        const Variant& v = st.variants[valid[i]];
        if (ws_bytes_of(v, *desc, OH, OW) > workspace_bytes) continue;
        if (ref_i < 0) ref_i = (int)i;
        if (v.split == 1 && v.family != FAM_WINOGRAD) {
            ref_i = (int)i;
            break;
        }
    }
    void* ref = nullptr;
    uint32_t* stats = nullptr;
    if (ref_i >= 0) {
        e = hipMalloc(&ref, out_bytes + 256);
        if (e == hipSuccess) e = hipMalloc((void**)&stats, 256);
        if (e != hipSuccess) {
            if (ref) (void)hipFree(ref);
            hipEventDestroy(e0);
            hipEventDestroy(e1);
            return hip_fail(e, "hipMalloc (autotune cross-check buffer)");
        }
        ConvArgs a;
        fill_args(a, *desc, OH, OW, in, filt, bias, out, workspace);
        status = run_variant(st.variants[valid[ref_i]], *desc, a, s);
        if (status == CONV_OK) {
            e = hipMemcpyAsync(ref, out, out_bytes, hipMemcpyDeviceToDevice, s);
            if (e != hipSuccess) status = hip_fail(e, "hipMemcpyAsync");
        }
    }
    const char* corrupt = getenv("CONVFWD_AUTOTUNE_CORRUPT");
    const double check_limit = desc->dtype == CONV_F32 ? 2e-5 : desc->dtype == CONV_F16 ? 5e-3 : 1e-2;
    for (size_t i = 0; i < valid.size() && status == CONV_OK; ++i) {
        const Variant& v = st.variants[valid[i]];
        const size_t need = ws_bytes_of(v, *desc, OH, OW);
        if (need > workspace_bytes) continue;
        ConvArgs a;
        fill_args(a, *desc, OH, OW, in, filt, bias, out, workspace);
        // warm-up, then a first timed launch pair to size the batch
        for (int w = 0; w < 2 && status == CONV_OK; ++w) status = run_variant(v, *desc, a, s);
        if (status) break;
        if (corrupt && v.name == corrupt) {
            // test hook (see include/convfwd.h): make this candidate's output wrong from the host side
            e = hipMemsetAsync(out, 0x7b, std::min<size_t>(out_bytes, 64), s);
            if (e != hipSuccess) {
                status = hip_fail(e, "hipMemsetAsync");
                break;
            }
        }
        if ((int)i != ref_i) {
            double err = 0.0;
            e = compare_outputs(desc->dtype, out, ref, n_out, stats, s, &err);
            if (e != hipSuccess) {
                status = hip_fail(e, "compare_outputs");
                break;
            }
            if (!(err <= check_limit)) {
                times[i] = -2.0;  // rejected: not timed, never selected
                continue;
            }
        }
        auto timed = [&](int reps, float& ms) -> int {
            hipError_t ee = hipEventRecord(e0, s);
            if (ee != hipSuccess) return hip_fail(ee, "hipEventRecord");
            for (int r = 0; r < reps; ++r) {
                const int rr = run_variant(v, *desc, a, s);
                if (rr) return rr;
            }
            ee = hipEventRecord(e1, s);
            if (ee != hipSuccess) return hip_fail(ee, "hipEventRecord");
            ee = hipEventSynchronize(e1);
            if (ee != hipSuccess) return hip_fail(ee, "hipEventSynchronize");
            ee = hipEventElapsedTime(&ms, e0, e1);
            if (ee != hipSuccess) return hip_fail(ee, "hipEventElapsedTime");
            return CONV_OK;
        };
        float ms = 0.f;
        status = timed(3, ms);
        if (status) break;
        const double est_us = std::max(1.0, ms * 1000.0 / 3.0);
        int reps = (int)std::min(100.0, std::max(5.0, 1500.0 / est_us));  // about 1.5 ms per batch
        double best_us = 1e30;
        for (int b = 0; b < 3 && status == CONV_OK; ++b) {
            status = timed(reps, ms);
            best_us = std::min(best_us, ms * 1000.0 / reps);
        }
        if (status) break;
        times[i] = best_us;
        if (best < 0 || best_us < times[best]) best = (int)i;
        if (need == 0 && (best_nows < 0 || best_us < times[best_nows])) best_nows = (int)i;
    }
    if (ref) {
        (void)hipStreamSynchronize(s);
        (void)hipFree(ref);
        (void)hipFree(stats);
    }
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    if (status) return status;
    if (best < 0) return CONV_EWORKSPACE;
    {
        std::lock_guard<std::mutex> g(st.mu);
        Choice c;
        c.best = st.variants[valid[best]].name;
        c.best_nows = best_nows >= 0 ? st.variants[valid[best_nows]].name : std::string();
        st.cache[key_of(*desc)] = c;
        st.times_us[key_of(*desc)] = times;
    }
    return CONV_OK;
}

int conv_compare_outputs(int32_t dtype, const void* got, const void* ref, size_t elements, void* stream, double* max_norm_err)
{
    if (dtype != CONV_F32 && dtype != CONV_F16 && dtype != CONV_BF16) return CONV_EDTYPE;
    if (!got || !ref || !max_norm_err || elements < 1 || elements >= ((size_t)1 << 31)) return CONV_EINVAL;
    uint32_t* stats = nullptr;
    hipError_t e = hipMalloc((void**)&stats, 256);
    if (e != hipSuccess) return hip_fail(e, "hipMalloc");
    e = compare_outputs(dtype, got, ref, elements, stats, (hipStream_t)stream, max_norm_err);
    (void)hipFree(stats);
    if (e != hipSuccess) return hip_fail(e, "compare_outputs");
    return CONV_OK;
}

int conv_variant_count(const conv_desc* desc)
{
    int OH, OW;
    const int rc = check_desc(desc, OH, OW);
    if (rc) return rc;
    State& st = state();
    std::lock_guard<std::mutex> g(st.mu);
    return (int)memo_of(st, *desc, OH, OW).valid.size();
}

int conv_variant_name(const conv_desc* desc, int idx, char* buf, size_t n)
{
    int OH, OW;
    const int rc = check_desc(desc, OH, OW);
    if (rc) return rc;
    if (!buf || n == 0) return CONV_EINVAL;
    State& st = state();
    std::lock_guard<std::mutex> g(st.mu);
    int reg;
    if (idx == -1 || idx == -2) {
        reg = select_variant(st, *desc, OH, OW, idx == -1 ? (size_t)-1 : 0);
        if (reg < 0) return reg;
    } else {
        const std::vector<int>& valid = memo_of(st, *desc, OH, OW).valid;
        if (idx < 0 || idx >= (int)valid.size()) return CONV_ENOVARIANT;
        reg = valid[idx];
    }
    snprintf(buf, n, "%s", st.variants[reg].name.c_str());
    return CONV_OK;
}

long long conv_variant_workspace(const conv_desc* desc, int idx)
{
    int OH, OW;
    const int rc = check_desc(desc, OH, OW);
    if (rc) return rc;
    State& st = state();
    std::lock_guard<std::mutex> g(st.mu);
    const std::vector<int>& valid = memo_of(st, *desc, OH, OW).valid;
    if (idx < 0 || idx >= (int)valid.size()) return CONV_ENOVARIANT;
    return (long long)ws_bytes_of(st.variants[valid[idx]], *desc, OH, OW);
}

int conv_force_variant(const conv_desc* desc, int idx)
{
    int OH, OW;
    const int rc = check_desc(desc, OH, OW);
    if (rc) return rc;
    State& st = state();
    std::lock_guard<std::mutex> g(st.mu);
    if (idx == -1) {
        st.forced.erase(key_of(*desc));
        return CONV_OK;
    }
    if (idx < 0 || idx >= (int)memo_of(st, *desc, OH, OW).valid.size()) return CONV_ENOVARIANT;
    st.forced[key_of(*desc)] = idx;
    return CONV_OK;
}

double conv_variant_time_us(const conv_desc* desc, int idx)
{
    int OH, OW;
    if (check_desc(desc, OH, OW)) return -1.0;
    State& st = state();
    std::lock_guard<std::mutex> g(st.mu);
    auto it = st.times_us.find(key_of(*desc));
    if (it == st.times_us.end() || idx < 0 || idx >= (int)it->second.size()) return -1.0;
    return it->second[idx];
}

int conv_cache_load(const char* path)
{
    if (!path) return CONV_EINVAL;
    std::ifstream f(path);
    if (!f) return CONV_EIO;
    State& st = state();
    std::map<Key, Choice> loaded;
    std::string line;
    while (std::getline(f, line)) {
        if (line.rfind("#! convfwd-cache", 0) == 0) {
            // identity line of a saved cache: measurements of another device model or another set of kernels are refused
            std::istringstream hs(line.substr(2));
            std::string tok, dev, reg;
            while (hs >> tok) {
                if (tok.rfind("device=", 0) == 0) dev = tok.substr(7);
                if (tok.rfind("registry=", 0) == 0) reg = tok.substr(9);
            }
            if (dev.empty() || reg.empty()) return CONV_EIO;
            const std::string here = device_id();
            if (reg != registry_id(st)) return CONV_EIO;
            if (dev != "none" && here != "none" && dev != here) return CONV_EIO;
            continue;
        }
        if (line.empty() || line[0] == '#') continue;
        // "N C H W K R S stride pad dtype flags | best | best_nows"
        std::vector<std::string> parts;
        size_t pos = 0;
        while (true) {
            size_t bar = line.find('|', pos);
            parts.push_back(line.substr(pos, bar == std::string::npos ? std::string::npos : bar - pos));
            if (bar == std::string::npos) break;
            pos = bar + 1;
        }
        if (parts.size() != 3) return CONV_EIO;
        std::istringstream ks(parts[0]);
        Key k;
        for (auto& x : k)
            if (!(ks >> x)) return CONV_EIO;
        std::string extra;
        if (ks >> extra) return CONV_EIO;
        auto trim = [](std::string s) {
            const size_t b = s.find_first_not_of(" \t\r"), e = s.find_last_not_of(" \t\r");
            return b == std::string::npos ? std::string() : s.substr(b, e - b + 1);
        };
        Choice c;
        c.best = trim(parts[1]);
        c.best_nows = trim(parts[2]);
        loaded[k] = c;
    }
    std::lock_guard<std::mutex> g(st.mu);
    for (auto& kv : loaded) {
        Choice c = kv.second;
        if (!st.by_name.count(c.best)) c.best.clear();
        if (!st.by_name.count(c.best_nows)) c.best_nows.clear();
        if (c.best.empty() && c.best_nows.empty()) continue;  // names from another build of the library
        st.cache[kv.first] = c;
    }
    return CONV_OK;
}

int conv_cache_save(const char* path)
{
    if (!path) return CONV_EINVAL;
    State& st = state();
    std::ofstream f(path);
    if (!f) return CONV_EIO;
    f << "#! convfwd-cache device=" << device_id() << " registry=" << registry_id(st) << "\n";
    f << "# convfwd autotune cache: N C H W K R S stride pad dtype flags | best | best without workspace\n";
    std::lock_guard<std::mutex> g(st.mu);
    for (auto& kv : st.cache) {
        for (size_t i = 0; i < kv.first.size(); ++i) f << (i ? " " : "") << kv.first[i];
        f << " | " << kv.second.best << " | " << kv.second.best_nows << "\n";
    }
    f.flush();
    return f ? CONV_OK : CONV_EIO;
}

void conv_cache_clear(void)
{
    State& st = state();
    std::lock_guard<std::mutex> g(st.mu);
    st.cache.clear();
    st.forced.clear();
    st.times_us.clear();
}

int conv_coop_load_plan(int threads, int words, int* loads_per_thread, int* last_load_guarded)
{
    if (threads < 1 || words < 1 || !loads_per_thread || !last_load_guarded) return CONV_EINVAL;
    const CoopPlan p = coop_plan(threads, words);
    *loads_per_thread = p.loads;
    *last_load_guarded = p.last_guarded ? 1 : 0;
    return CONV_OK;
}

int maxpool_fwd(int32_t N, int32_t C, int32_t H, int32_t W, int32_t win, int32_t stride, int32_t dtype, const void* in,
                void* out, void* stream)
{
    if (dtype != CONV_F32 && dtype != CONV_F16 && dtype != CONV_BF16) return CONV_EDTYPE;
    if (N < 1 || C < 1 || H < 1 || W < 1 || win < 1 || stride < 1 || win > H || win > W || !in || !out)
        return CONV_EINVAL;
    if ((double)N * C * (double)H * W >= 2147483648.0) return CONV_EINVAL;
    const hipError_t e = launch_maxpool(N, C, H, W, win, stride, dtype, false, false, in, out, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e, "maxpool");
    return CONV_OK;
}

int maxpool_fwd_layout(int32_t N, int32_t C, int32_t H, int32_t W, int32_t win, int32_t stride, int32_t dtype,
                       int32_t in_nhwc, int32_t out_nhwc, const void* in, void* out, void* stream)
{
    if (dtype != CONV_F32 && dtype != CONV_F16 && dtype != CONV_BF16) return CONV_EDTYPE;
    if (N < 1 || C < 1 || H < 1 || W < 1 || win < 1 || stride < 1 || win > H || win > W || !in || !out)
        return CONV_EINVAL;
    if ((double)N * C * (double)H * W >= 2147483648.0) return CONV_EINVAL;
    const hipError_t e =
        launch_maxpool(N, C, H, W, win, stride, dtype, in_nhwc != 0, out_nhwc != 0, in, out, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e, "maxpool");
    return CONV_OK;
}

int conv_convert_layout(int32_t A, int32_t B, int32_t S, int32_t dtype, const void* in, void* out, void* stream)
{
    if (dtype != CONV_F32 && dtype != CONV_F16 && dtype != CONV_BF16) return CONV_EDTYPE;
    if (A < 1 || B < 1 || S < 1 || A > 65535 || !in || !out || in == out) return CONV_EINVAL;
    if ((double)A * B * (double)S >= 2147483648.0 || (S + 31) / 32 > 2147483647 || (B + 31) / 32 > 65535) return CONV_EINVAL;
    const hipError_t e = launch_transpose(A, B, S, dtype_size(dtype), in, out, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e, "convert_layout");
    return CONV_OK;
}

// The target format of a filter conversion: the flag the descriptor carries, else Winograd for fp32 and the MFMA
// operand order for the 16-bit types.
static uint32_t filter_target(const conv_desc* desc)
{
    if (desc->flags & CONV_FLAG_FILT_PACKED) return CONV_FLAG_FILT_PACKED;
    if (desc->flags & CONV_FLAG_FILT_WINOGRAD) return CONV_FLAG_FILT_WINOGRAD;
    return desc->dtype == CONV_F32 ? CONV_FLAG_FILT_WINOGRAD : CONV_FLAG_FILT_PACKED;
}

int conv_run_ops(const conv_op* ops, int32_t count, void* stream, int32_t* failed_index)
{
    if (!ops || count < 0) return CONV_EINVAL;
    for (int32_t i = 0; i < count; ++i) {
        const conv_op& o = ops[i];
        int rc;
        switch (o.kind) {
            case CONV_OP_CONV:
                rc = fwd_common(&o.desc, o.in, o.filt, o.bias, o.out, o.workspace, o.workspace_bytes, stream);
                break;
            case CONV_OP_MAXPOOL:
                rc = maxpool_fwd_layout(o.p[0], o.p[1], o.p[2], o.p[3], o.p[4], o.p[5], o.p[6], o.p[7], o.p[8], o.in, o.out, stream);
                break;
            case CONV_OP_CONVERT:
                rc = conv_convert_layout(o.p[0], o.p[1], o.p[2], o.p[3], o.in, o.out, stream);
                break;
            default:
                rc = CONV_EINVAL;
        }
        if (rc != CONV_OK) {
            if (failed_index) *failed_index = i;
            return rc;
        }
    }
    return CONV_OK;
}

size_t conv_transformed_filter_bytes(const conv_desc* desc)
{
    int OH, OW;
    if (check_desc(desc, OH, OW)) return 0;
    if ((desc->flags & CONV_FLAG_FILT_PACKED) && (desc->flags & CONV_FLAG_FILT_WINOGRAD)) return 0;
    State& st = state();
    if (filter_target(desc) == CONV_FLAG_FILT_PACKED) {
        // served when some packed-filter kernel accepts the layer with a channel-innermost input
        if (desc->dtype == CONV_F32 || (desc->C % 16) != 0 || (desc->flags & CONV_FLAG_FILT_KRSC)) return 0;
        conv_desc d = *desc;
        d.flags = (d.flags & ~(kLayoutFlags | CONV_FLAG_MAXPOOL_3X3S2)) | CONV_FLAG_FILT_PACKED | CONV_FLAG_IN_NHWC;
        std::lock_guard<std::mutex> g(st.mu);
        if (memo_of(st, d, OH, OW).valid.empty()) return 0;
        return (size_t)((d.K + 31) / 32) * 32 * (size_t)d.C * d.R * d.S * 2;
    }
    conv_desc d = *desc;
    d.flags = (d.flags & ~kLayoutFlags) | CONV_FLAG_FILT_WINOGRAD;
    if (desc->flags & kLayoutFlags) return 0;
    std::lock_guard<std::mutex> g(st.mu);
    if (memo_of(st, d, OH, OW).valid.empty()) return 0;
    return wino_transformed_filter_bytes(d.K, d.C);
}

int conv_transform_filters(const conv_desc* desc, const void* filt, void* out, void* stream)
{
    int OH, OW;
    const int rc = check_desc(desc, OH, OW);
    if (rc) return rc;
    if (!filt || !out || !aligned16(filt) || (((uintptr_t)out) & 255u) || filt == out) return CONV_EINVAL;
    if (conv_transformed_filter_bytes(desc) == 0) return CONV_ENOVARIANT;
    hipError_t e;
    if (filter_target(desc) == CONV_FLAG_FILT_PACKED)
        e = launch_pack_filters16(filt, out, desc->K, desc->C, desc->R * desc->S, (hipStream_t)stream);
    else
        e = launch_wino_filter_transform((const float*)filt, (float*)out, desc->K, desc->C, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e, "transform_filters");
    return CONV_OK;
}

int conv_probe_mfma_peak(int32_t dtype, int32_t block, void* scratch, void* stream, double* tflops)
{
    if (dtype != CONV_F32 && dtype != CONV_F16 && dtype != CONV_BF16) return CONV_EDTYPE;
    if ((block != 16 && block != 32) || !scratch || !tflops) return CONV_EINVAL;
    const hipError_t e = probe_mfma(dtype, block, (float*)scratch, (hipStream_t)stream, tflops);
    if (e != hipSuccess) return hip_fail(e, "probe_mfma");
    return CONV_OK;
}

int conv_probe_mfma_mix(int32_t dtype, int32_t block, int32_t waves_per_simd, int32_t valu_per_mfma,
                        int32_t distinct_operands, void* scratch, void* stream, double* tflops, double* ns_per_mfma)
{
    if (dtype != CONV_F32 && dtype != CONV_F16 && dtype != CONV_BF16) return CONV_EDTYPE;
    if ((block != 16 && block != 32) || !scratch || !tflops || !ns_per_mfma) return CONV_EINVAL;
    if (waves_per_simd < 1 || waves_per_simd > 4) return CONV_EINVAL;
    if (valu_per_mfma != 0 && valu_per_mfma != 2 && valu_per_mfma != 4 && valu_per_mfma != 8) return CONV_EINVAL;
    if (distinct_operands && (valu_per_mfma != 0 || dtype == CONV_F32)) return CONV_EINVAL;
    const hipError_t e = probe_mfma_mix(dtype, block, waves_per_simd, valu_per_mfma, distinct_operands, (float*)scratch, (hipStream_t)stream,
                                        tflops, ns_per_mfma);
    if (e != hipSuccess) return hip_fail(e, "probe_mfma_mix");
    return CONV_OK;
}

int conv_probe_stream_bandwidth(const void* src, void* dst, size_t bytes, void* stream, double* gbytes_per_s)
{
    if (!src || !dst || bytes < 16 || !gbytes_per_s || !aligned16(src) || !aligned16(dst)) return CONV_EINVAL;
    const hipError_t e = probe_copy(src, dst, bytes, (hipStream_t)stream, gbytes_per_s);
    if (e != hipSuccess) return hip_fail(e, "probe_copy");
    return CONV_OK;
}

const char* conv_strerror(int status)
{
    thread_local std::string buf;
    switch (status) {
        case CONV_OK: return "success";
        case CONV_EINVAL: return "invalid descriptor, pointer, alignment or size";
        case CONV_EDTYPE: return "unsupported dtype";
        case CONV_EWORKSPACE:
            if (g_ws_msg.empty()) return "workspace missing or too small";
            buf = "workspace missing or too small: " + g_ws_msg;
            g_ws_msg.clear();
            return buf.c_str();
        case CONV_EHIP: buf = "HIP error: " + g_hip_msg; return buf.c_str();
        case CONV_ENOVARIANT: return "no such variant for this descriptor";
        case CONV_EIO: return "autotune cache file unreadable, unwritable or malformed";
        default: return "unknown status";
    }
}

}  // extern "C"
