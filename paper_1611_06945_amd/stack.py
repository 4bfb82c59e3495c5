"""A fixed sequence of convolution layers with max-pools in between, run through the C ABI.

The paper's execution model for a compute graph (Section 3, "Code Generation,
Scheduling, and Execution"): every ND-Array is allocated up front, the operations
are issued in a topological order on one stream, and the outputs stay on the GPU.
Here the graph is a straight line, so the order is the list order.  PyTorch only
provides the device buffers; every operation is a call into libconvfwd.so.

The stack can also apply the paper's second graph-level optimisation (Section 3,
"Graph-level Optimizations"): choosing a data format per operation and inserting
the conversions.  With `formats="auto"` every layer that has a channel-innermost
kernel (fp16/bf16, C % 8 == 0, K % 8 == 0) is timed in both formats, the
conversions are timed, and the cheapest assignment over the whole chain is found
by dynamic programming.  A max-pool between two layers converts for free (it reads
one layout and writes the other); elsewhere an explicit conversion is inserted.
Filters of channel-innermost layers are repacked once in `prepare()`: either
[K][R][S][C], or the matrix-instruction operand order of the packed-filter
kernels ("nhwc_packed"), whichever measures faster for the layer.  The stack's
input and final output are always [N][C][H][W].

Where a max-pool follows a layer whose kernels can pool their own output tile
(CONV_FLAG_MAXPOOL_3X3S2: the paper's fusion rule applied to the pooling
operation), the fused call replaces convolution + pool when `fuse_pool` asks for
it, or, with `formats="auto"`, when it measures faster.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

from . import binding as B
from .workloads import ConvShape

NCHW, NHWC = "nchw", "nhwc"
NHWC_PACKED = "nhwc_packed"   # a layer format: channel-innermost activations, filters in MFMA operand order
KCRS, KRSC, PACKED = "kcrs", "krsc", "packed"


class ConvStack:
    def __init__(self, shapes: Sequence[ConvShape], dtype: int, pool_after: Sequence[int] = (), relu: bool = True,
                 pool_win: int = 3, pool_stride: int = 2, formats=None, fuse_pool: bool = False):
        """`pool_after` holds 1-based layer numbers that are followed by a max-pool.  `formats`: None = every layer
        in [N][C][H][W]; "auto" = decided by autotune(); or a list of "nchw"/"nhwc", one per layer.  `fuse_pool`: pool
        inside the convolution wherever a kernel can (with "auto" the timings decide instead).  A list entry may also be
        "nhwc_packed": channel-innermost activations with the filters in MFMA operand order."""
        import torch

        self.torch = torch
        self.shapes = list(shapes)
        self.dtype = dtype
        self.relu = relu
        self.pool_after = set(pool_after)
        self.pool_win, self.pool_stride = pool_win, pool_stride
        self.tdt = {B.CONV_F32: torch.float32, B.CONV_F16: torch.float16, B.CONV_BF16: torch.bfloat16}[dtype]
        n = len(self.shapes)
        for i in range(n - 1):
            got = self._pooled_shape(i) if (i + 1) in self.pool_after else self.shapes[i].out_shape()
            want = self.shapes[i + 1].in_shape()
            if tuple(got) != tuple(want):
                raise ValueError("layer %d produces %s but layer %d expects %s" % (i + 1, tuple(got), i + 2, want))
        self.auto = formats == "auto"
        given = [NCHW] * n if formats in (None, "auto") else list(formats)
        if len(given) != n or any(f not in (NCHW, NHWC, NHWC_PACKED) for f in given):
            raise ValueError("formats must name nchw, nhwc or nhwc_packed for each of the %d layers" % n)
        self.formats = [NHWC if f == NHWC_PACKED else f for f in given]                     # activation layout per layer
        self.filt_formats = [{NCHW: KCRS, NHWC: KRSC, NHWC_PACKED: PACKED}[f] for f in given]  # filter format per layer
        for i, f in enumerate(self.formats):
            if f == NHWC and not self.nhwc_capable(i):
                raise ValueError("layer %d has no channel-innermost kernel" % (i + 1))
            if self.filt_formats[i] == PACKED and not self.packed_capable(i):
                raise ValueError("layer %d has no packed-filter kernel" % (i + 1))
        self.packed_filts: List[Optional[object]] = [None] * n
        self.plan_times = None
        self.out_layouts = None   # set by the format selection: the output layout it timed and chose per layer
        self.fused = [bool(fuse_pool) and self.can_fuse_pool(i, self.formats[i], self._handoff_layout(i)) for i in range(n)]
        self._build()

    # ---- geometry --------------------------------------------------------------------------------------------------
    def nhwc_capable(self, i: int) -> bool:
        s = self.shapes[i]
        return self.dtype != B.CONV_F32 and s.C % 8 == 0 and s.K % 8 == 0

    def packed_capable(self, i: int) -> bool:
        d = B.desc_of(self.shapes[i], self.dtype, relu=self.relu, in_nhwc=True, filt_packed=True)
        return self.dtype != B.CONV_F32 and B.conv_variant_count(d) > 0

    def _desc(self, i: int, fmt: str, filt_fmt: str, out_nhwc: bool, maxpool: bool = False):
        return B.desc_of(self.shapes[i], self.dtype, relu=self.relu, in_nhwc=fmt == NHWC, out_nhwc=out_nhwc,
                         filt_krsc=filt_fmt == KRSC, filt_packed=filt_fmt == PACKED, maxpool=maxpool)

    def _pooled_shape(self, i: int):
        s = self.shapes[i]
        oh = (s.OH - self.pool_win) // self.pool_stride + 1
        ow = (s.OW - self.pool_win) // self.pool_stride + 1
        return (s.N, s.K, oh, ow)

    def _handoff_layout(self, i: int) -> str:
        """Layout of what layer i hands on: what the next layer consumes; [N][C][H][W] after the last layer."""
        return self.formats[i + 1] if i + 1 < len(self.shapes) else NCHW

    def planar_writes_nhwc(self, i: int) -> bool:
        """Whether a kernel for planar input can write layer i's output channel-innermost (first-layer window kernels)."""
        if self.dtype == B.CONV_F32:
            return False
        d = B.desc_of(self.shapes[i], self.dtype, relu=self.relu, out_nhwc=True)
        return B.conv_variant_count(d) > 0

    def can_fuse_pool(self, i: int, fmt: str, out_layout: str) -> bool:
        """Whether some kernel runs layer i in format `fmt` with the following 3x3 stride-2 pool fused, writing `out_layout`."""
        if (i + 1) not in self.pool_after or (self.pool_win, self.pool_stride) != (3, 2):
            return False
        d = self._desc(i, fmt, KRSC if fmt == NHWC else KCRS, out_layout == NHWC, maxpool=True)
        return B.conv_variant_count(d) > 0

    def _conv_out_layout(self, i: int) -> str:
        """A channel-innermost kernel writes whatever layout is wanted next; the planar kernels write [N][K][OH][OW],
        except those that can write channel-innermost when that is what is wanted next.  When a pool follows a
        channel-innermost layer, the pool converts, so the convolution keeps the layout of its own format."""
        if self.fused[i]:
            return self._handoff_layout(i)   # the fused call writes the pooled tensor, in the layout wanted next
        if self.out_layouts is not None:
            return self.out_layouts[i]
        if self.formats[i] == NCHW:
            return NHWC if self._handoff_layout(i) == NHWC and self.planar_writes_nhwc(i) else NCHW
        return NHWC if (i + 1) in self.pool_after else self._handoff_layout(i)

    def _build(self) -> None:
        torch = self.torch
        self._ops_key = None
        n = len(self.shapes)
        self.descs, self.conv_out, self.pool_out, self.conv_layout, self.convert_out = [], [], [], [], []
        ws_bytes = 256
        for i, s in enumerate(self.shapes):
            lay = self._conv_out_layout(i)
            if self.fused[i] and self.filt_formats[i] == PACKED:
                self.filt_formats[i] = KRSC   # only the [K][R][S][C] kernels pool their own tile
            d = self._desc(i, self.formats[i], self.filt_formats[i], lay == NHWC, maxpool=self.fused[i])
            self.descs.append(d)
            self.conv_layout.append(lay)
            # buffers are flat in memory; the shape recorded here is the logical [N][K][OH][OW] one
            self.conv_out.append(None if self.fused[i] else torch.empty(s.out_shape(), dtype=self.tdt, device="cuda"))
            self.pool_out.append(torch.empty(self._pooled_shape(i), dtype=self.tdt, device="cuda")
                                 if (i + 1) in self.pool_after else None)
            # an explicit conversion is needed only where no pool follows and the layouts differ
            need_cvt = self.pool_out[i] is None and lay != self._handoff_layout(i)
            self.convert_out.append(torch.empty(s.out_shape(), dtype=self.tdt, device="cuda") if need_cvt else None)
            ws_bytes = max(ws_bytes, B.conv_workspace_bytes(d))
        self.in_convert = (torch.empty(self.shapes[0].in_shape(), dtype=self.tdt, device="cuda")
                           if self.formats[0] == NHWC else None)
        self.workspace = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")

    def layer_output(self, i: int):
        """What layer i (0-based) hands to the next one (device tensor, in layout `output_layout(i)`)."""
        if self.pool_out[i] is not None:
            return self.pool_out[i]
        return self.convert_out[i] if self.convert_out[i] is not None else self.conv_out[i]

    def output_layout(self, i: int) -> str:
        return self._handoff_layout(i)

    # ---- one-time preparation ----------------------------------------------------------------------------------------
    def prepare(self, filts, stream=None) -> None:
        """Repack the filters of channel-innermost layers ([K][C][R][S] -> [K][R][S][C], or -> MFMA operand order); done
        once, not per run."""
        for i, s in enumerate(self.shapes):
            if self.filt_formats[i] == KRSC:
                self.packed_filts[i] = self.torch.empty_like(filts[i])
                B.conv_convert_layout(s.K, s.C, s.R * s.S, self.dtype, filts[i], self.packed_filts[i], stream)
            elif self.filt_formats[i] == PACKED:
                nbytes = B.conv_transformed_filter_bytes(self.descs[i])
                self.packed_filts[i] = self.torch.empty(nbytes // 2, dtype=self.torch.int16, device="cuda")
                B.conv_transform_filters(self.descs[i], filts[i], self.packed_filts[i], stream)
            else:
                self.packed_filts[i] = None

    def _filt(self, i: int, filts):
        if self.filt_formats[i] != KCRS:
            if self.packed_filts[i] is None:
                raise RuntimeError("prepare(filts) must run before a stack with channel-innermost layers")
            return self.packed_filts[i]
        return filts[i]

    # ---- execution ---------------------------------------------------------------------------------------------------
    def _after_conv(self, i: int, stream) -> None:
        s = self.shapes[i]
        if self.fused[i]:
            return
        if self.pool_out[i] is not None:
            B.maxpool_fwd_layout(s.N, s.K, s.OH, s.OW, self.pool_win, self.pool_stride, self.dtype,
                                 self.conv_layout[i] == NHWC, self._handoff_layout(i) == NHWC, self.conv_out[i],
                                 self.pool_out[i], stream)
        elif self.convert_out[i] is not None:
            if self.conv_layout[i] == NCHW:   # -> channel-innermost
                B.conv_convert_layout(s.N, s.K, s.OH * s.OW, self.dtype, self.conv_out[i], self.convert_out[i], stream)
            else:
                B.conv_convert_layout(s.N, s.OH * s.OW, s.K, self.dtype, self.conv_out[i], self.convert_out[i], stream)

    def _first_input(self, x, stream):
        if self.in_convert is None:
            return x
        s = self.shapes[0]
        B.conv_convert_layout(s.N, s.C, s.H * s.W, self.dtype, x, self.in_convert, stream)
        return self.in_convert

    def _walk(self, x, filts, biases, stream, tune: bool):
        cur = self._first_input(x, stream)
        for i, d in enumerate(self.descs):
            call = B.conv_autotune if tune else B.conv_fwd_ws
            out = self.pool_out[i] if self.fused[i] else self.conv_out[i]
            call(d, cur, self._filt(i, filts), biases[i], out, self.workspace, self.workspace.numel(), stream)
            self._after_conv(i, stream)
            cur = self.layer_output(i)
        return cur

    def _ops(self, x, filts, biases):
        """The whole chain as an array of library operations (built once per set of tensors, then reused)."""
        key = (int(x.data_ptr()), tuple(int(f.data_ptr()) for f in filts), tuple(0 if b is None else int(b.data_ptr()) for b in biases),
               tuple(0 if p is None else int(p.data_ptr()) for p in self.packed_filts), id(self.workspace))
        if getattr(self, "_ops_key", None) == key:
            return self._ops_arr
        ops = []
        cur = x
        if self.in_convert is not None:
            s0 = self.shapes[0]
            ops.append(B.op_convert(s0.N, s0.C, s0.H * s0.W, self.dtype, x, self.in_convert))
            cur = self.in_convert
        for i, d in enumerate(self.descs):
            s = self.shapes[i]
            out = self.pool_out[i] if self.fused[i] else self.conv_out[i]
            ops.append(B.op_conv(d, cur, self._filt(i, filts), biases[i], out, self.workspace, self.workspace.numel()))
            if not self.fused[i]:
                if self.pool_out[i] is not None:
                    ops.append(B.op_maxpool(s.N, s.K, s.OH, s.OW, self.pool_win, self.pool_stride, self.dtype,
                                            self.conv_layout[i] == NHWC, self._handoff_layout(i) == NHWC, self.conv_out[i],
                                            self.pool_out[i]))
                elif self.convert_out[i] is not None:
                    dims = (s.N, s.K, s.OH * s.OW) if self.conv_layout[i] == NCHW else (s.N, s.OH * s.OW, s.K)
                    ops.append(B.op_convert(*dims, self.dtype, self.conv_out[i], self.convert_out[i]))
            cur = self.layer_output(i)
        self._ops_arr = (B.conv_op * len(ops))(*ops)
        self._ops_key = key
        return self._ops_arr

    def run(self, x, filts, biases, stream=None):
        """Enqueue every operation with one call into the library (`conv_run_ops`: the chain is issued from native code,
        not paced by a Python call per kernel); returns the last layer's output tensor, [N][K][OH][OW] (not
        synchronised)."""
        B.conv_run_ops(self._ops(x, filts, biases), stream)
        return self.layer_output(len(self.shapes) - 1)

    def run_stepwise(self, x, filts, biases, stream=None):
        """The same chain issued one binding call per operation (what `run` did before the native schedule existed)."""
        return self._walk(x, filts, biases, stream, tune=False)

    def capture(self, x, filts, biases):
        """Record one run of the stack (every convolution, pool and conversion, on the given tensors) into a HIP graph
        by stream capture and return it; `graph.replay()` then launches the whole chain with one call.  Variants must be
        selected (autotune or cache) before: the captured launches are those of the selection at capture time.  The
        result of a replay is in the same buffers as after `run` (`layer_output(len(shapes) - 1)`)."""
        torch = self.torch
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            self.run(x, filts, biases)      # once outside the capture: kernel attributes are set on a first launch
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.run(x, filts, biases)
        return graph

    def autotune(self, x, filts, biases, stream=None) -> None:
        """Autotune every layer on real data; with formats="auto", first choose the formats."""
        if self.auto:
            self._choose_formats(x, filts, biases, stream)
        self.prepare(filts, stream)
        self._walk(x, filts, biases, stream, tune=True)

    # ---- format selection --------------------------------------------------------------------------------------------
    def _time_op(self, fn, reps: int = 20) -> float:
        """Microseconds per call of a pool or conversion on the device.  The calls are recorded into a HIP graph and the
        replay is timed: enqueued one by one from Python they would take longer to issue than to run.  `fn` must issue
        on the current stream (stream=None): that is the stream the capture records."""
        torch = self.torch
        fn()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for _ in range(reps):
                fn()
        graph.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        graph.replay()
        e1.record()
        e1.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / reps
        if not us > 0.0:
            raise RuntimeError("timed an empty graph: the operation was not issued on the capturing stream")
        return us

    def _choose_formats(self, x, filts, biases, stream) -> None:
        """Time each layer in each format (its best variant), each conversion and each pool, then pick per layer by
        dynamic programming over the chain, on scratch tensors filled with random values."""
        torch = self.torch
        n = len(self.shapes)
        conv_t = [{} for _ in range(n)]      # (format, out layout) -> microseconds (the faster filter format)
        filt_pick = [{} for _ in range(n)]   # (format, out layout) -> the filter format that gave it
        fused_t = [{} for _ in range(n)]     # (format, pooled-output layout) -> microseconds of convolution + fused pool
        glue_t = [{} for _ in range(n)]      # (conv out layout, handoff layout) -> microseconds of pool / conversion
        for i, s in enumerate(self.shapes):
            # random values of the size of real activations and weights: kernels run measurably faster on zeros
            xin = torch.rand(s.in_shape(), device="cuda").to(self.tdt)
            f = (torch.randn(s.filt_shape(), device="cuda") * (2.0 / (s.C * s.R * s.S)) ** 0.5).to(self.tdt)
            out = torch.empty(s.out_shape(), dtype=self.tdt, device="cuda")
            for fmt in ((NCHW, NHWC) if self.nhwc_capable(i) else (NCHW,)):
                ffmts = (KCRS,) if fmt == NCHW else ((KRSC, PACKED) if self.packed_capable(i) else (KRSC,))
                for olay in ((NCHW, NHWC) if fmt == NHWC or self.planar_writes_nhwc(i) else (NCHW,)):
                    for ff in ffmts:
                        d = self._desc(i, fmt, ff, olay == NHWC)
                        if B.conv_variant_count(d) == 0:
                            continue
                        # timing only: the kernels' run time does not depend on which filter values sit where
                        fbuf = f if ff != PACKED else torch.zeros(B.conv_transformed_filter_bytes(d) // 2, dtype=torch.int16,
                                                                  device="cuda")
                        if ff == PACKED:
                            B.conv_transform_filters(d, f, fbuf, stream)
                        ws = torch.empty(max(256, B.conv_workspace_bytes(d)), dtype=torch.uint8, device="cuda")
                        B.conv_autotune(d, xin, fbuf, biases[i], out, ws, ws.numel(), stream)
                        t = B.conv_time_us(d, xin, fbuf, biases[i], out, ws, ws.numel(), stream, launches=20)
                        if t < conv_t[i].get((fmt, olay), float("inf")):
                            conv_t[i][(fmt, olay)] = t
                            filt_pick[i][(fmt, olay)] = ff
            pooled = (i + 1) in self.pool_after
            dst = torch.empty(self._pooled_shape(i) if pooled else s.out_shape(), dtype=self.tdt, device="cuda")
            for fmt in ((NCHW, NHWC) if self.nhwc_capable(i) else (NCHW,)):
                for olay in (NCHW, NHWC):
                    if not self.can_fuse_pool(i, fmt, olay):
                        continue
                    d = self._desc(i, fmt, KRSC if fmt == NHWC else KCRS, olay == NHWC, maxpool=True)
                    ws = torch.empty(max(256, B.conv_workspace_bytes(d)), dtype=torch.uint8, device="cuda")
                    B.conv_autotune(d, xin, f, biases[i], dst, ws, ws.numel(), stream)
                    fused_t[i][(fmt, olay)] = B.conv_time_us(d, xin, f, biases[i], dst, ws, ws.numel(), stream, launches=20)
            for a in (NCHW, NHWC):
                for b in (NCHW, NHWC):
                    if pooled:
                        glue_t[i][(a, b)] = self._time_op(lambda: B.maxpool_fwd_layout(
                            s.N, s.K, s.OH, s.OW, self.pool_win, self.pool_stride, self.dtype, a == NHWC, b == NHWC, out, dst))
                    elif a == b:
                        glue_t[i][(a, b)] = 0.0
                    else:
                        dims = (s.N, s.K, s.OH * s.OW) if a == NCHW else (s.N, s.OH * s.OW, s.K)
                        glue_t[i][(a, b)] = self._time_op(lambda: B.conv_convert_layout(*dims, self.dtype, out, dst))
        s0 = self.shapes[0]
        x_scratch = torch.empty_like(x)
        x_cvt = self._time_op(lambda: B.conv_convert_layout(
            s0.N, s0.C, s0.H * s0.W, self.dtype, x, x_scratch)) if self.nhwc_capable(0) else float("inf")
        chosen, olays, fused, total = plan_formats(conv_t, fused_t, glue_t, x_cvt)
        self.plan_times = {"conv_us": conv_t, "glue_us": glue_t, "fused_pool_us": fused_t, "input_convert_us": x_cvt,
                           "total_us": total}
        self.formats = chosen
        self.out_layouts = olays
        self.fused = fused
        self.filt_formats = [(KRSC if chosen[i] == NHWC else KCRS) if fused[i] else filt_pick[i][(chosen[i], olays[i])]
                             for i in range(n)]
        self._build()


def plan_formats(conv_t, fused_t, glue_t, x_cvt):
    """The cheapest assignment of data formats over a chain of layers, by dynamic programming (pure host logic).

    conv_t[i][(fmt, olay)]: microseconds of layer i run in format `fmt` writing layout `olay`; fused_t[i][(fmt, olay)]:
    the same with the following pool computed by the convolution (`olay` is then the pooled tensor's layout);
    glue_t[i][(olay, want)]: microseconds of what turns layout `olay` into the layout `want` handed to layer i + 1 (the
    pool behind layer i, which converts on the way, or an explicit conversion; 0 where nothing is needed); x_cvt: the
    conversion of the stack's planar input to channel-innermost (inf if layer 0 has no such kernel).  The last layer
    hands on [N][C][H][W].  Returns (format per layer, output layout per layer, pool fused per layer, total)."""
    n = len(conv_t)
    # best[i][fmt] = cheapest time of layers 0..i-1 plus glue, arriving at layer i with its input in layout fmt
    best = [{NCHW: 0.0, NHWC: x_cvt}]
    back = []
    for i in range(n):
        nxt, bk = {}, {}
        for want in (NCHW, NHWC):            # layout handed on after layer i
            if i == n - 1 and want != NCHW:
                continue
            for (fmt, olay), t in conv_t[i].items():
                # a pool converts from olay to `want`; without a pool the kernel may write `want` itself
                total = best[i].get(fmt, float("inf")) + t + glue_t[i][(olay, want)]
                if total < nxt.get(want, float("inf")):
                    nxt[want], bk[want] = total, (fmt, olay, False)
            for (fmt, olay), t in fused_t[i].items():
                total = best[i].get(fmt, float("inf")) + t
                if olay == want and total < nxt.get(want, float("inf")):
                    nxt[want], bk[want] = total, (fmt, olay, True)
        best.append(nxt)
        back.append(bk)
    if NCHW not in best[n]:
        raise ValueError("no assignment of formats serves the chain")
    want, chosen, olays, fused = NCHW, [None] * n, [None] * n, [False] * n
    for i in range(n - 1, -1, -1):
        fmt, olay, fz = back[i][want]
        chosen[i], olays[i], fused[i] = fmt, olay, fz
        want = fmt
    return chosen, olays, fused, best[n][NCHW]
