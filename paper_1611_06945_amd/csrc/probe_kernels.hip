// Measured ceilings of the device the library runs on: an MFMA issue loop per storage type and a streaming copy.
// They give the bench a measured denominator next to the published peaks (sustained clocks differ from the datasheet).
#include "igemm_kernel.h"

namespace convfwd {

// Every wave keeps NACC independent accumulator blocks and issues `iters` rounds of MFMAs on them: no memory traffic,
// no dependency between consecutive instructions.  flops = waves * iters * NACC * flops_per_mfma.
template <int DT, int MB, int NACC>
__global__ __launch_bounds__(256) void mfma_loop_kernel(float* sink, int iters, float seed)
{
    typedef Mma<DT, MB> mma_t;
    typedef typename mma_t::acc_t acc_t;
    acc_t acc[NACC];
#pragma unroll
    for (int i = 0; i < NACC; ++i)
        for (int v = 0; v < (int)(sizeof(acc_t) / sizeof(float)); ++v) acc[i][v] = 0.0f;
    if constexpr (DT == CONV_F32) {
        const float a = seed + threadIdx.x, b = seed * 0.5f;
        for (int it = 0; it < iters; ++it)
#pragma unroll
            for (int i = 0; i < NACC; ++i) acc[i] = mma_t::run(a, b, acc[i]);
    } else {
        const uint32_t w = __builtin_bit_cast(uint32_t, seed) | 0x3c003c00u;
        const uint4 a = make_uint4(w, w, w, w), b = make_uint4(w ^ 1u, w, w, w);
        for (int it = 0; it < iters; ++it)
#pragma unroll
            for (int i = 0; i < NACC; ++i) acc[i] = mma_t::run(a, b, acc[i]);
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < NACC; ++i) s += acc[i][0];
    if (s == 123.456f) sink[0] = s;  // keeps the loop alive without a store on the normal path
}

// The same loop with a chosen number of waves per SIMD and, optionally, NV vector-ALU instructions between consecutive
// MFMAs: one workgroup of 256 * WPS threads per CU (the launch asks for the whole LDS so that no second workgroup fits),
// so every SIMD holds exactly WPS waves.  Answers two questions the kernels are built around: how much of the issue
// rate one wave per SIMD reaches on its own, and whether vector-ALU work overlaps with MFMA work of the same SIMD.
template <int DT, int MB, int NACC, int NV, int OPM = 0>
__global__ void mfma_mix_kernel(float* sink, int iters, float seed)
{
    typedef Mma<DT, MB> mma_t;
    typedef typename mma_t::acc_t acc_t;
    acc_t acc[NACC];
#pragma unroll
    for (int i = 0; i < NACC; ++i)
        for (int v = 0; v < (int)(sizeof(acc_t) / sizeof(float)); ++v) acc[i][v] = 0.0f;
    float x[NV > 0 ? NV : 1];
#pragma unroll
    for (int j = 0; j < (NV > 0 ? NV : 1); ++j) x[j] = seed + (float)(threadIdx.x + j);
    const uint32_t w = __builtin_bit_cast(uint32_t, seed) | 0x3c003c00u;
    const uint4 a16 = make_uint4(w, w, w, w), b16 = make_uint4(w ^ 1u, w, w, w);
    const float a32 = seed + threadIdx.x, b32 = seed * 0.5f;
    // OPM: 0 = every MFMA reads the same two operand registers; 1 = a different B operand per MFMA; 2 = different A and B
    // (16-bit types; what a real kernel does)
    uint4 av[NACC], bv[NACC];
#pragma unroll
    for (int i = 0; i < NACC; ++i) {
        av[i] = make_uint4(w + i, w, w ^ threadIdx.x, w);
        bv[i] = make_uint4(w, w + 2 * i, w, w ^ threadIdx.x);
        asm volatile("" : "+v"(av[i].x), "+v"(av[i].y), "+v"(av[i].z), "+v"(av[i].w));
        asm volatile("" : "+v"(bv[i].x), "+v"(bv[i].y), "+v"(bv[i].z), "+v"(bv[i].w));
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < NACC; ++i) {
            if constexpr (DT == CONV_F32)
                acc[i] = mma_t::run(a32, b32, acc[i]);
            else if constexpr (OPM == 0)
                acc[i] = mma_t::run(a16, b16, acc[i]);
            else if constexpr (OPM == 1)
                acc[i] = mma_t::run(a16, bv[i], acc[i]);
            else
                acc[i] = mma_t::run(av[i], bv[i], acc[i]);
#pragma unroll
            for (int j = 0; j < NV; ++j) asm volatile("v_fma_f32 %0, %0, %1, %0" : "+v"(x[j]) : "v"(b32));
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < NACC; ++i) s += acc[i][0];
#pragma unroll
    for (int j = 0; j < (NV > 0 ? NV : 1); ++j) s += x[j];
    if (s == 123.456f) sink[0] = s;
}

template <int DT, int MB, int NV, int OPM = 0, int NACC_ = 0>
static hipError_t time_mfma_mix(int wps, float* sink, hipStream_t s, double* tflops, double* cycles_hint)
{
    constexpr int NACC = NACC_ ? NACC_ : (MB == 32 ? 4 : 8);
    const int iters = 2048;
    const void* fn = (const void*)mfma_mix_kernel<DT, MB, NACC, NV, OPM>;
    hipError_t e = ensure_dynamic_lds(fn, 160 * 1024);
    if (e != hipSuccess) return e;
    hipEvent_t e0, e1;
    e = hipEventCreate(&e0);
    if (e != hipSuccess) return e;
    e = hipEventCreate(&e1);
    if (e != hipSuccess) {
        hipEventDestroy(e0);
        return e;
    }
    float best = 1e30f;
    for (int rep = 0; rep < 4 && e == hipSuccess; ++rep) {
        hipEventRecord(e0, s);
        hipLaunchKernelGGL((mfma_mix_kernel<DT, MB, NACC, NV, OPM>), dim3(256), dim3(256 * wps), 160 * 1024, s, sink, iters, 1.0f);
        e = hipGetLastError();
        hipEventRecord(e1, s);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (rep > 0 && ms < best) best = ms;
    }
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    if (e != hipSuccess) return e;
    const double kdepth = DT == CONV_F32 ? (MB == 32 ? 2.0 : 4.0) : (MB == 32 ? 16.0 : 32.0);
    const double mfmas_per_simd = (double)wps * iters * NACC;
    *tflops = 256.0 * 4.0 * mfmas_per_simd * 2.0 * MB * MB * kdepth / (best * 1e-3) / 1e12;
    *cycles_hint = best * 1e-3 / mfmas_per_simd * 1e9;  // nanoseconds per MFMA and SIMD
    return hipSuccess;
}

template <int DT, int MB>
static hipError_t mix_by_nv(int nv, int distinct, int wps, float* sink, hipStream_t s, double* tflops, double* ns)
{
    if (distinct) return nv == 0 ? time_mfma_mix<DT, MB, 0, 2>(wps, sink, s, tflops, ns) : hipErrorInvalidValue;
    switch (nv) {
        case 0: return time_mfma_mix<DT, MB, 0>(wps, sink, s, tflops, ns);
        case 2: return time_mfma_mix<DT, MB, 2>(wps, sink, s, tflops, ns);
        case 4: return time_mfma_mix<DT, MB, 4>(wps, sink, s, tflops, ns);
        case 8: return time_mfma_mix<DT, MB, 8>(wps, sink, s, tflops, ns);
        default: return hipErrorInvalidValue;
    }
}

hipError_t probe_mfma_mix(int dtype, int block, int wps, int nv, int distinct, float* sink, hipStream_t s, double* tflops, double* ns)
{
    if (block == 32) {
        if (dtype == CONV_F32) return mix_by_nv<CONV_F32, 32>(nv, distinct, wps, sink, s, tflops, ns);
        if (dtype == CONV_F16) return mix_by_nv<CONV_F16, 32>(nv, distinct, wps, sink, s, tflops, ns);
        return mix_by_nv<CONV_BF16, 32>(nv, distinct, wps, sink, s, tflops, ns);
    }
    if (dtype == CONV_F32) return mix_by_nv<CONV_F32, 16>(nv, distinct, wps, sink, s, tflops, ns);
    if (dtype == CONV_F16) return mix_by_nv<CONV_F16, 16>(nv, distinct, wps, sink, s, tflops, ns);
    return mix_by_nv<CONV_BF16, 16>(nv, distinct, wps, sink, s, tflops, ns);
}

__global__ __launch_bounds__(256) void stream_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

template <int DT, int MB>
static hipError_t time_mfma(float* sink, hipStream_t s, double* tflops)
{
    constexpr int NACC = MB == 32 ? 4 : 8;
    const int iters = 4096, wgs = 256 * 8;
    hipEvent_t e0, e1;
    hipError_t e = hipEventCreate(&e0);
    if (e != hipSuccess) return e;
    e = hipEventCreate(&e1);
    if (e != hipSuccess) {
        hipEventDestroy(e0);
        return e;
    }
    float best = 1e30f;
    for (int rep = 0; rep < 4 && e == hipSuccess; ++rep) {
        hipEventRecord(e0, s);
        hipLaunchKernelGGL((mfma_loop_kernel<DT, MB, NACC>), dim3(wgs), dim3(256), 0, s, sink, iters, 1.0f);
        e = hipGetLastError();
        hipEventRecord(e1, s);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (rep > 0 && ms < best) best = ms;
    }
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    if (e != hipSuccess) return e;
    const double kdepth = DT == CONV_F32 ? (MB == 32 ? 2.0 : 4.0) : (MB == 32 ? 16.0 : 32.0);
    const double flops = (double)wgs * 4.0 * iters * NACC * 2.0 * MB * MB * kdepth;
    *tflops = flops / (best * 1e-3) / 1e12;
    return hipSuccess;
}

hipError_t probe_mfma(int dtype, int block, float* sink, hipStream_t s, double* tflops)
{
    if (block == 32) {
        if (dtype == CONV_F32) return time_mfma<CONV_F32, 32>(sink, s, tflops);
        if (dtype == CONV_F16) return time_mfma<CONV_F16, 32>(sink, s, tflops);
        return time_mfma<CONV_BF16, 32>(sink, s, tflops);
    }
    if (dtype == CONV_F32) return time_mfma<CONV_F32, 16>(sink, s, tflops);
    if (dtype == CONV_F16) return time_mfma<CONV_F16, 16>(sink, s, tflops);
    return time_mfma<CONV_BF16, 16>(sink, s, tflops);
}

hipError_t probe_copy(const void* src, void* dst, size_t bytes, hipStream_t s, double* gbs)
{
    const size_t n = bytes / 16;
    hipEvent_t e0, e1;
    hipError_t e = hipEventCreate(&e0);
    if (e != hipSuccess) return e;
    e = hipEventCreate(&e1);
    if (e != hipSuccess) {
        hipEventDestroy(e0);
        return e;
    }
    float best = 1e30f;
    for (int rep = 0; rep < 5 && e == hipSuccess; ++rep) {
        hipEventRecord(e0, s);
        hipLaunchKernelGGL(stream_copy_kernel, dim3(256 * 16), dim3(256), 0, s, (const uint4*)src, (uint4*)dst, n);
        e = hipGetLastError();
        hipEventRecord(e1, s);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (rep > 0 && ms < best) best = ms;
    }
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    if (e != hipSuccess) return e;
    *gbs = 2.0 * (double)(n * 16) / (best * 1e-3) / 1e9;  // bytes read + bytes written
    return hipSuccess;
}

}  // namespace convfwd
