/*
 * convfwd.h -- C ABI of the MI355X (gfx950) forward-convolution library.
 *
 * The operation is the convolution layer the paper defines in Section 2
 * ("Background": output = conv(input, filters); each output value is the dot
 * product of one filter with a window of the input slid with a spatial stride)
 * with the activation fused into the output write as in Section 3
 * ("Graph-level Optimizations"), plus a per-output-channel bias:
 *
 *   out[n,k,oy,ox] = act( bias[k] + sum_{c,r,s} in[n,c,oy*stride-pad+r,ox*stride-pad+s]
 *                                                * filt[k,c,r,s] )
 *
 * zero padding, no filter flip, OH = floor((H+2*pad-R)/stride)+1 (OW likewise;
 * floor reproduces the in->out sizes of Appendix A), groups = 1, dilation = 1.
 *
 * Conventions shared by every entry point
 *   - Tensors are dense, C order: in [N][C][H][W], filt [K][C][R][S],
 *     out [N][K][OH][OW], element type `dtype` (fp32, or fp16/bf16 storage with
 *     fp32 accumulation and one round-to-nearest-even on the store).
 *   - `bias` is [K] fp32 or NULL (= no bias); it is added in fp32 before `act`.
 *   - All tensor pointers are DEVICE pointers owned by the caller.  The library
 *     reads in/filt/bias, writes out (which must not alias them), keeps no pointer
 *     after returning, never allocates or frees device memory and never
 *     synchronises, except conv_autotune() which times kernels and therefore
 *     synchronises `stream`.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Kernels are enqueued on it and the call returns immediately.
 *   - Return value: 0 on success, a negative conv_status otherwise.  Descriptor
 *     and pointer validation happens before the first HIP call, so the error
 *     paths work on a host without a GPU.
 *   - Thread safety: the variant cache is guarded by a mutex; kernels hold no state.
 */
#ifndef CONVFWD_H
#define CONVFWD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { CONV_F32 = 0, CONV_F16 = 1, CONV_BF16 = 2 } conv_dtype; /* storage type of in/filt/out */

enum {
    CONV_FLAG_RELU = 1u,      /* act = max(x,0); without it act is the identity */
    /* Optional channel-innermost formats (the paper's explicit data-format conversions, Section 3 "Graph-level
     * Optimizations"): the same operation on tensors stored as in [N][H][W][C], filt [K][R][S][C], out [N][OH][OW][K].
     * Kernels exist for fp16/bf16 with IN_NHWC and FILT_KRSC both set, C % 8 == 0 (and K % 8 == 0 with OUT_NHWC) and
     * an input and a filter tensor below 1 GiB each,
     * and, with OUT_NHWC alone (planar input and filters, channel-innermost output), for the fp16/bf16 first layers the
     * strided window kernels serve (3 channels, 11x11 stride 4 or 7x7 stride 2; K % 4 == 0): the conversion then costs
     * nothing.  Any other combination of these bits gives CONV_ENOVARIANT.  conv_convert_layout() converts tensors. */
    CONV_FLAG_IN_NHWC = 2u,
    CONV_FLAG_OUT_NHWC = 4u,
    CONV_FLAG_FILT_KRSC = 8u,
    /* Filters handed over in the Winograd F(2x2,3x3) domain, as written by conv_transform_filters() for the same
     * descriptor (without this bit): at inference the weights are constants, so the filter transform is one of the
     * conversions the paper does ahead of time (Section 3, "Graph-level Optimizations").  Only the Winograd variants
     * serve such a descriptor (fp32, 3x3, stride 1, pad <= 1, C % 8 == 0; otherwise CONV_ENOVARIANT), and they then
     * need no workspace.  Not combinable with the channel-innermost bits. */
    CONV_FLAG_FILT_WINOGRAD = 16u,
    /* A 3x3 stride-2 max-pool (no padding, the pooling layers of the paper's networks) fused behind the activation:
     * out holds [N][K][PH][PW] (or [N][PH][PW][K] with OUT_NHWC), PH = (OH-3)/2 + 1, PW = (OW-3)/2 + 1, each element
     * the maximum of act(conv + bias) over its window -- the convolution's own output is never written (the paper's
     * rule for fusing an operation into the write of the convolution result, Section 3 "Graph-level Optimizations").
     * Needs OH, OW >= 3.  Served by the window kernels whose workgroup holds a whole output image (stride 1; fp16/bf16:
     * OH*OW <= 192 for 3x3 and 5x5 windows, <= 768 for 5x5 channel-innermost; fp32: 3x3 windows, OH*OW <= 208, planar
     * tensors), and for fp16/bf16 first layers (C = 3; 11x11 stride 4 or 7x7 stride 2; any image size; planar input,
     * pooled output in either format, K % 8 == 0 for the channel-innermost one) by a kernel whose workgroups compute tiles
     * of pooled outputs; other descriptors give CONV_ENOVARIANT and the caller
     * runs maxpool_fwd() behind the convolution.  The result is bit-identical to that sequence run with the same
     * variant (for the first-layer kernel: with a kernel that sums in the same order), NaN sums included (with the activation they become 0 before the pool, as in the sequence; without it a
     * NaN in the window is the result); only the sign of a zero result can differ when the activation is the identity.
     * Not combinable with CONV_FLAG_FILT_WINOGRAD. */
    CONV_FLAG_MAXPOOL_3X3S2 = 32u,
    /* Filters handed over in the order the 16-bit matrix instructions consume them, as written by
     * conv_transform_filters() for the same descriptor with this bit set: the other ahead-of-time filter conversion
     * (Section 3, "Graph-level Optimizations"; the filter operand then goes from memory straight into the multiplying
     * wave's registers).  fp16/bf16, stride 1, C % 16 == 0, windows the packed-filter kernels are built for (3x3,
     * 5x5) with pad < window, input channel-innermost (CONV_FLAG_IN_NHWC), output in either format; otherwise
     * CONV_ENOVARIANT.  Not combinable with CONV_FLAG_FILT_KRSC, CONV_FLAG_FILT_WINOGRAD or CONV_FLAG_MAXPOOL_3X3S2. */
    CONV_FLAG_FILT_PACKED = 64u
};

typedef enum {
    CONV_OK = 0,
    CONV_EINVAL = -1,     /* NULL descriptor/pointer; N,C,H,W,K,R,S < 1; stride < 1; pad < 0; window larger than
                             the padded input; a tensor with 2^31 or more elements or 4 GiB or more; a tensor pointer
                             that is not 16-byte aligned; unknown flag bits */
    CONV_EDTYPE = -2,     /* dtype is not one of conv_dtype */
    CONV_EWORKSPACE = -3, /* workspace NULL/too small for what was asked (forced split variant, autotune) */
    CONV_EHIP = -4,       /* a HIP call failed; conv_strerror(CONV_EHIP) carries the HIP message */
    CONV_ENOVARIANT = -5, /* variant index out of range, or no kernel accepts this descriptor */
    CONV_EIO = -6         /* autotune-cache file could not be read or written, or is malformed */
} conv_status;

typedef struct {
    int32_t N, C, H, W;   /* input batch, channels, height, width            */
    int32_t K, R, S;      /* output channels, window height, window width    */
    int32_t stride, pad;  /* same stride and symmetric zero pad on both axes */
    int32_t dtype;        /* conv_dtype                                      */
    uint32_t flags;       /* CONV_FLAG_*                                     */
} conv_desc;

/* Extent of the tensor the call writes: (OH, OW) by the formula above, or (PH, PW) with CONV_FLAG_MAXPOOL_3X3S2.
 * Pure host code.  CONV_EINVAL if the descriptor is not valid. */
int conv_out_shape(const conv_desc* desc, int32_t* OH, int32_t* OW);

/* FLOPs of the layer in the convention of Appendix A: 2*N*K*OH*OW*C*R*S.  0 if the descriptor is invalid. */
double conv_flops(const conv_desc* desc);

/*
 * Bytes of device workspace with which every variant valid for `desc` can run
 * (split-reduction variants keep fp32 partial sums there, the Winograd variants
 * the transformed filters).  conv_fwd() needs none.  Returns 0 for an invalid
 * descriptor.
 */
size_t conv_workspace_bytes(const conv_desc* desc);

/*
 * Enqueue the fused convolution on `stream` using the variant selected for
 * `desc` (forced > autotuned/cached > heuristic), restricted to variants that
 * need no workspace.  Asynchronous; see the conventions above.
 */
int conv_fwd(const conv_desc* desc, const void* in, const void* filt, const float* bias, void* out,
             void* stream);

/*
 * As conv_fwd, but may also pick a variant that needs scratch memory (paper,
 * Section 3 "Variant Selection and Autotuning": several variants per
 * operation): a split-reduction variant, whose partial sums go to `workspace`
 * (device memory, 256-byte aligned, contents undefined afterwards) and are then
 * reduced in a fixed order, or, for fp32 3x3 stride-1 layers, a Winograd
 * F(2x2,3x3) variant (the algorithm the paper names as its main open topic,
 * Section 4 "Experimental Results"), which first writes the transformed filters
 * there.  Results are bit-reproducible either way.  If `workspace_bytes` is too small for the selected variant
 * the best variant that fits is used instead; CONV_EWORKSPACE only if a forced
 * variant does not fit.
 */
int conv_fwd_ws(const conv_desc* desc, const void* in, const void* filt, const float* bias, void* out,
                void* workspace, size_t workspace_bytes, void* stream);

/*
 * For callers that cannot allocate device memory or be handed a workspace (code under HIP graph capture, serving
 * loops, harnesses that forbid hipMalloc): conv_fwd_ws with the scratch memory taken from an array the library holds
 * itself, CONV_STATIC_SCRATCH_BYTES per GPU, resident from library load to process end.  The call allocates and frees
 * nothing.  The variant is selected as conv_fwd_ws selects it with unlimited workspace (forced > autotuned/cached >
 * cost model); when that variant needs more than CONV_STATIC_SCRATCH_BYTES the call is rejected with CONV_EWORKSPACE
 * (conv_strerror names the variant and both sizes) and nothing is enqueued -- use conv_fwd or conv_fwd_ws then.
 * Results are bit-identical to conv_fwd_ws running the same variant.  Nothing in the array has to start at zero
 * (every partial sum and every transformed filter is written before it is read), and its contents are undefined
 * afterwards.  Every call on one GPU shares that GPU's array: calls that overlap in time on one GPU (different
 * streams, or threads) race on it and must be serialised by the caller; calls on one stream are ordered.
 */
#define CONV_STATIC_SCRATCH_BYTES (32u << 20)
int conv_fwd_static(const conv_desc* desc, const void* in, const void* filt, const float* bias, void* out,
                    void* stream);

/*
 * Brute-force autotuning (paper, Section 3 "Variant Selection and Autotuning":
 * exhaustive search over a fixed set of configurations, by measured run time):
 * runs every variant valid for `desc` that fits `workspace_bytes` on the given
 * buffers, times it with device events on `stream`, and records the fastest in
 * the in-process cache used by conv_fwd/conv_fwd_ws (two entries: best overall,
 * best without workspace).  `out` is overwritten.  Synchronises `stream`.
 * `workspace` may be NULL (then only variants without workspace are tried).
 * Every candidate's output is cross-checked before it may win (the paper's tuning flow verifies outputs numerically,
 * Section 4 "Experimental Setup"): the output of a reference candidate (the first unsplit direct variant that fits)
 * is kept, and a candidate whose output differs from it by more than 2e-5 (fp32), 5e-3 (fp16) or 1e-2 (bf16: one
 * rounding step of an 8-bit significand) in the max-normalised sense of conv_compare_outputs() is neither timed nor
 * selected; conv_variant_time_us() then reports -2 for it.  For this check -- and only here -- the call allocates and
 * frees a temporary device buffer of the size of `out`.  Test hook: when the environment variable
 * CONVFWD_AUTOTUNE_CORRUPT names a variant, the first bytes of that candidate's output are overwritten from the host
 * before the check, so that the rejection path can be exercised without a wrong kernel.
 */
int conv_autotune(const conv_desc* desc, const void* in, const void* filt, const float* bias, void* out,
                  void* workspace, size_t workspace_bytes, void* stream);

/* Number of variants valid for `desc` (negative conv_status on error).  Pure host code. */
int conv_variant_count(const conv_desc* desc);

/*
 * Name of variant `idx` in [0, conv_variant_count) -- or, with idx = -1, of the
 * variant conv_fwd_ws would pick now given unlimited workspace; idx = -2, of the
 * one conv_fwd would pick -- copied NUL-terminated into buf[0..n).  Names read
 * like the paper's tuning strings, e.g. "igemm_f32_M128N128K16_w2x2" or "..._sk4".
 */
int conv_variant_name(const conv_desc* desc, int idx, char* buf, size_t n);

/* Workspace bytes variant `idx` of `desc` needs (0 for unsplit direct variants); negative conv_status on error. */
long long conv_variant_workspace(const conv_desc* desc, int idx);

/* Force variant `idx` for this exact descriptor in later conv_fwd/conv_fwd_ws calls (tests run every variant this
 * way); idx = -1 removes the override. */
int conv_force_variant(const conv_desc* desc, int idx);

/* Last measured time (microseconds per launch) of variant `idx` from conv_autotune in this process; -1 if it was not
 * tried (no autotune yet, or it did not fit the workspace), -2 if the cross-check rejected its output. */
double conv_variant_time_us(const conv_desc* desc, int idx);

/*
 * Device-side time of the currently selected variant (the one conv_fwd_ws would run with this workspace): `launches`
 * back-to-back launches on `stream`, bracketed by two events; *us_per_launch = elapsed / launches.  This is the paper's
 * measurement rule (Section 4, "Experimental Results": device timers around the calls, host overheads excluded), used
 * by the benchmark for layers whose run time is of the order of a host-side launch.  Synchronises the stream.
 * Pointers, alignment and errors as conv_fwd_ws; launches >= 1 and us_per_launch != NULL, else CONV_EINVAL.
 */
int conv_time_us(const conv_desc* desc, const void* in, const void* filt, const float* bias, void* out, void* workspace,
                 size_t workspace_bytes, void* stream, int launches, double* us_per_launch);

/*
 * The error metric of the parity tests and of the autotuner's cross-check on two device tensors of `elements`
 * elements of `dtype`: max_i |got_i - ref_i| / max(max_j |ref_j|, 1e-30); infinity if `got` holds a NaN, or an
 * infinity where `ref` is finite (the paper compares outputs with relative tolerances, Section 4 "Experimental
 * Setup").  Synchronises `stream`; allocates 256 bytes of device scratch for the duration of the call.
 */
int conv_compare_outputs(int32_t dtype, const void* got, const void* ref, size_t elements, void* stream,
                         double* max_norm_err);

/*
 * Autotune cache persistence: a text file, one line per descriptor
 * ("N C H W K R S stride pad dtype flags | best-name | best-no-workspace-name").
 * A saved file starts with an identity line ("#! convfwd-cache device=<arch/name/CUs> registry=<hash of the
 * library's variant list>"): measurements are only valid for the device model and the set of kernels they were
 * taken with, so load refuses (CONV_EIO) a file whose identity line names another registry, or another device
 * when both sides know theirs ("none" = written or read on a host without a GPU); a file without an identity line
 * (hand-written) is accepted.  Load merges into the in-process cache and ignores lines naming unknown
 * variants; a missing, unreadable or malformed file gives CONV_EIO and leaves
 * the cache as it was.  conv_cache_clear drops every cached and forced choice.
 */
int conv_cache_load(const char* path);
int conv_cache_save(const char* path);
void conv_cache_clear(void);

/*
 * Cooperative tile load plan (paper, Section 3 "Metaprogramming for NN
 * Convolutions": `threads` threads loading `words` words need ceil(words/threads)
 * loads each, and only the last one needs a bounds guard, and only when `words`
 * is not a multiple of `threads`).  The tile loaders of the kernels are unrolled
 * from the same rule at compile time; this host entry point exposes it for
 * checking.  CONV_EINVAL if either count is < 1.
 */
int conv_coop_load_plan(int threads, int words, int* loads_per_thread, int* last_load_guarded);

/*
 * Per-channel spatial max-pool, window win x win, stride `stride`, no padding,
 * OH = floor((H-win)/stride)+1 (the glue between layers of a convolution stack;
 * paper, Section 2).  in [N][C][H][W] -> out [N][C][OH][OW], element type
 * `dtype`, device pointers, asynchronous on `stream`.  On every path (either layout, and the pool fused into a
 * convolution without activation) the window is scanned row by row, the first of equal values is kept (so the sign
 * of a zero is that of the first zero) and a NaN anywhere in the window is the result.
 */
int maxpool_fwd(int32_t N, int32_t C, int32_t H, int32_t W, int32_t win, int32_t stride, int32_t dtype,
                const void* in, void* out, void* stream);

/* The same pooling on either tensor layout: in_nhwc / out_nhwc != 0 means channel-innermost ([N][H][W][C]) for that
 * side, 0 means [N][C][H][W].  With different layouts on the two sides it is also the format conversion between two
 * layers.  Errors as maxpool_fwd. */
int maxpool_fwd_layout(int32_t N, int32_t C, int32_t H, int32_t W, int32_t win, int32_t stride, int32_t dtype,
                       int32_t in_nhwc, int32_t out_nhwc, const void* in, void* out, void* stream);

/*
 * A straight-line schedule of operations issued with ONE call (paper, Section 3 "Code Generation, Scheduling, and
 * Execution": every ND-Array is allocated up front and the operations are issued in a topological order): each
 * element is a conv_fwd_ws, maxpool_fwd_layout or conv_convert_layout call with its arguments, and conv_run_ops
 * enqueues them in array order on `stream` exactly as those calls would -- same validation, same variant selection,
 * same kernels -- without returning to the caller in between, so that a chain of microsecond kernels is not paced by
 * the caller's own per-call cost.  Stops at the first element that fails and returns its status (*failed_index, if not
 * NULL, receives its index; earlier elements stay enqueued); CONV_EINVAL for a NULL array, count < 0 or an unknown kind.
 *   kind CONV_OP_CONV:    desc, in, filt, bias, out, workspace, workspace_bytes as conv_fwd_ws
 *   kind CONV_OP_MAXPOOL: in, out; p[0..8] = N, C, H, W, win, stride, dtype, in_nhwc, out_nhwc as maxpool_fwd_layout
 *   kind CONV_OP_CONVERT: in, out; p[0..3] = A, B, S, dtype as conv_convert_layout
 */
typedef enum { CONV_OP_CONV = 0, CONV_OP_MAXPOOL = 1, CONV_OP_CONVERT = 2 } conv_op_kind;
typedef struct {
    int32_t kind;           /* conv_op_kind */
    conv_desc desc;         /* CONV_OP_CONV only */
    const void* in;
    const void* filt;       /* CONV_OP_CONV only */
    const float* bias;      /* CONV_OP_CONV only; may be NULL */
    void* out;
    void* workspace;        /* CONV_OP_CONV only; may be NULL */
    size_t workspace_bytes;
    int32_t p[9];           /* CONV_OP_MAXPOOL / CONV_OP_CONVERT parameters */
} conv_op;
int conv_run_ops(const conv_op* ops, int32_t count, void* stream, int32_t* failed_index);

/*
 * Explicit data-format conversion (paper, Section 3, "Graph-level Optimizations"): out[a][s][b] = in[a][b][s] for
 * dense tensors of `dtype` elements.  (A,B,S) = (N,C,H*W) turns [N][C][H][W] into [N][H][W][C]; (N,H*W,C) turns it
 * back; (K,C,R*S) turns filters [K][C][R][S] into [K][R][S][C].  Device pointers, out must not alias in; enqueued on
 * `stream`.  CONV_EINVAL for NULL/aliased pointers, extents < 1, A > 65535 or 2^31 or more elements.
 */
int conv_convert_layout(int32_t A, int32_t B, int32_t S, int32_t dtype, const void* in, void* out, void* stream);

/*
 * Ahead-of-time filter conversions as explicit, separately timed calls (paper, Section 3 "Graph-level
 * Optimizations": data-format conversions are operations of their own).  `filt` is the KCRS filter tensor (device,
 * 16-byte aligned); the result goes to `out` (device, 256-byte aligned, conv_transformed_filter_bytes(desc) bytes,
 * layout private to the library), which is then passed as `filt` of the layer's descriptor with the format's bit set.
 * The target format is the one whose bit `desc` carries:
 *   CONV_FLAG_FILT_WINOGRAD  U = G g G^T of the Winograd F(2x2,3x3) variants (fp32);
 *   CONV_FLAG_FILT_PACKED    the matrix-instruction operand order of the packed-filter kernels (fp16/bf16);
 * with neither bit it is the Winograd domain for fp32 and the packed order for fp16/bf16.  Other bits of `desc`
 * describe the layer as usual.  conv_transformed_filter_bytes returns 0, conv_transform_filters CONV_ENOVARIANT, when
 * no kernel of that format serves the layer; CONV_EINVAL for NULL or misaligned pointers.  Enqueued on `stream`.
 */
size_t conv_transformed_filter_bytes(const conv_desc* desc);
int conv_transform_filters(const conv_desc* desc, const void* filt, void* out, void* stream);

/*
 * Measured ceilings of the device, for reporting next to the published peaks (the paper's own practice of timing on
 * the device with device-level timers, Section 4 "Experimental Setup").  All synchronise `stream`.
 *  - conv_probe_mfma_peak: TFLOP/s of a register-only MFMA issue loop for `dtype` with 16x16 or 32x32 blocks
 *    (`block` = 16 or 32); `scratch` is any 4-byte device location (never written in practice).
 *  - conv_probe_stream_bandwidth: GB/s (bytes read + bytes written) of a plain copy of `bytes` from `src` to `dst`,
 *    both device pointers, 16-byte aligned, not overlapping.
 *  - conv_probe_mfma_mix: the same issue loop with exactly `waves_per_simd` (1..4) waves on every SIMD and
 *    `valu_per_mfma` (0, 2, 4 or 8) vector-ALU instructions between consecutive MFMAs: how much of the issue rate a
 *    given occupancy reaches, and whether vector-ALU work hides behind matrix work.  With `distinct_operands` != 0
 *    (16-bit types, valu_per_mfma = 0) every MFMA of a round reads operand registers of its own, as a real kernel
 *    does, instead of one shared pair.  Writes TFLOP/s and the nanoseconds one SIMD spends per MFMA.
 */
int conv_probe_mfma_peak(int32_t dtype, int32_t block, void* scratch, void* stream, double* tflops);
int conv_probe_mfma_mix(int32_t dtype, int32_t block, int32_t waves_per_simd, int32_t valu_per_mfma,
                        int32_t distinct_operands, void* scratch, void* stream, double* tflops, double* ns_per_mfma);
int conv_probe_stream_bandwidth(const void* src, void* dst, size_t bytes, void* stream, double* gbytes_per_s);

/* Text for a conv_status; for CONV_EHIP it includes the message of the last failed HIP call of this thread. */
const char* conv_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* CONVFWD_H */
