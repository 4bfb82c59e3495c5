#!/usr/bin/env python3
"""Forward-convolution benchmark on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-layers] [--no-cpu]

A step is one call of the fused convolution (conv_fwd_ws through the C ABI: filter-tile and patch-tile staging,
MFMA main loop, fused bias+ReLU store; plus the fixed-order reduce when a split variant is selected) on one
batch of seeded synthetic input that is already resident in device memory.  The variant is chosen by the
library's autotuner before timing starts.  The headline workload is the mid-network 3x3 layer of the batch
sweep at batch 20 in fp32 (the paper's arithmetic); `layers` in the JSON line reports every benchmark layer at
batch 1/5/20 and every storage type: ms, GFLOP/s and the fraction of the MFMA and HBM rooflines.

Every timed output is checked after the timed region against the CPU oracle on a seeded sample of output elements
(checker leg only; a figure whose output fails the check aborts the run).  `--format nhwc|nhwc_packed` runs the
16-bit layers on channel-innermost tensors (with the filters in MFMA operand order for nhwc_packed): the explicit
ahead-of-time conversions are timed separately and reported beside the layer.  `--probe` prints the device
microbenchmarks the kernel designs rest on instead of running a workload.

Prints ONE JSON line on stdout; everything else goes to stderr.
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X published peaks
PEAK_TFLOPS = {"f32": 157.3, "f16": 2500.0, "bf16": 2500.0}
PEAK_HBM_GBS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def all_workloads():
    from paper_1611_06945_amd import workloads as wl

    ws = [wl.config1(), wl.config2(), wl.config3()]
    for dt in (wl.F32, wl.F16, wl.BF16):
        for n in (1, 5, 20):
            ws.append(wl.config4(n, dt))
    ws += wl.config5_layers(20, wl.F16)
    return ws


TOL = {"f32": 1e-5, "f16": 5e-3, "bf16": 5e-3}   # max normalised error allowed per storage type


def executed_mfma_flops(variant, shape):
    """FLOPs the matrix units execute per call: the direct count, except for the Winograd variants, which multiply
    2.25x less (on tiles padded to the workgroup shape)."""
    import re

    m = re.match(r"wino_f32_M(\d+)T(\d+)_", variant)
    if not m:
        return float(shape.flops)
    tm, tt = int(m.group(1)), int(m.group(2))
    tiles = shape.N * ((shape.OH + 1) // 2) * ((shape.OW + 1) // 2)
    return 2.0 * 16 * (-(-shape.K // tm) * tm) * (-(-tiles // tt) * tt) * shape.C


class Resident:
    """A workload with its tensors in device memory (optionally several rotating copies), in one of three formats:
    "nchw" (the plain contract: [N][C][H][W], [K][C][R][S]), "nhwc" (channel-innermost tensors, filters [K][R][S][C]) or
    "nhwc_packed" (channel-innermost tensors, filters in MFMA operand order).  The conversions of the latter two are
    explicit library calls made here once, timed, and reported as `convert_us`.  "nchw_pool" is the plain contract with
    the 3x3 stride-2 max-pool computed by the convolution kernel (CONV_FLAG_MAXPOOL_3X3S2): the output is the pooled
    tensor, channel-innermost (what the next layer of the stack reads)."""

    def __init__(self, w, copies=1, fmt="nchw"):
        import numpy as np
        import torch

        from paper_1611_06945_amd import binding as B
        from paper_1611_06945_amd import workloads as wl

        self.w, self.B, self.torch, self.fmt = w, B, torch, fmt
        s = w.shape
        self.pool = fmt == "nchw_pool"
        nh = fmt in ("nhwc", "nhwc_packed")
        self.out_nhwc = nh or self.pool
        self.desc = B.desc_of(s, w.dtype, relu=True, in_nhwc=nh, out_nhwc=self.out_nhwc, filt_krsc=fmt == "nhwc",
                              filt_packed=fmt == "nhwc_packed", maxpool=self.pool)
        if B.conv_variant_count(self.desc) <= 0:
            raise ValueError("no kernel serves %s in format %s" % (w.name, fmt))
        self.data = data = w.generate()
        tdt = {wl.F32: torch.float32, wl.F16: torch.float16, wl.BF16: torch.bfloat16}[w.dtype]

        def up(a):
            if w.dtype == wl.BF16:
                return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
            return torch.from_numpy(a).cuda()

        self.convert_us = None
        x0, f0 = up(data["in"]), up(data["filt"])
        if nh:
            def timed(fn):
                fn()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(20):
                    fn()
                e1.record()
                e1.synchronize()
                return round(e0.elapsed_time(e1) * 1e3 / 20, 2)

            x1 = torch.empty((s.N, s.H, s.W, s.C), dtype=tdt, device="cuda")
            t_in = timed(lambda: B.conv_convert_layout(s.N, s.C, s.H * s.W, w.dtype, x0, x1))
            if fmt == "nhwc":
                f1 = torch.empty((s.K, s.R, s.S, s.C), dtype=tdt, device="cuda")
                t_f = timed(lambda: B.conv_convert_layout(s.K, s.C, s.R * s.S, w.dtype, f0, f1))
            else:
                f1 = torch.empty(B.conv_transformed_filter_bytes(self.desc) // 2, dtype=torch.int16, device="cuda")
                t_f = timed(lambda: B.conv_transform_filters(self.desc, f0, f1))
            self.convert_us = {"input_to_nhwc": t_in, "filters": t_f,
                               "note": "explicit conversions, host-enqueued one by one (includes launch gaps); in a stack the "
                                       "previous layer writes channel-innermost directly and filters convert once"}
            x0, f0 = x1, f1
        self.oh, self.ow = B.conv_out_shape(self.desc)   # pooled extent with the fused pool
        oshape = (s.N, self.oh, self.ow, s.K) if self.out_nhwc else (s.N, s.K, self.oh, self.ow)
        self.sets = []
        for _ in range(copies):
            self.sets.append((x0.clone(), f0.clone(), torch.from_numpy(data["bias"]).cuda(),
                              torch.full(oshape, float("nan"), dtype=tdt, device="cuda")))
        self.ws_bytes = max(256, B.conv_workspace_bytes(self.desc))
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device="cuda")
        self.i = 0

    def autotune(self):
        x, f, b, o = self.sets[0]
        self.B.conv_autotune(self.desc, x, f, b, o, self.ws, self.ws_bytes)
        self.variant = self.B.conv_variant_name(self.desc, -1)
        return self.variant

    def step(self):
        x, f, b, o = self.sets[self.i]
        self.i = (self.i + 1) % len(self.sets)
        self.B.conv_fwd_ws(self.desc, x, f, b, o, self.ws, self.ws_bytes)

    def time_device(self, launches, batches):
        """Median and minimum device-side time per launch (ms): the library issues the launches itself between two
        events, so the host-side cost of a Python call does not bound the figure for microsecond kernels."""
        x, f, b, o = self.sets[0]
        per = [self.B.conv_time_us(self.desc, x, f, b, o, self.ws, self.ws_bytes, launches=launches) * 1e-3
               for _ in range(batches)]
        return statistics.median(per), min(per)

    def time_batches(self, launches, batches, warmup):
        """Median and minimum time per launch (ms) over `batches` event-bracketed batches of `launches` launches."""
        torch = self.torch
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        per = []
        for _ in range(batches):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(launches):
                self.step()
            e1.record()
            e1.synchronize()
            per.append(e0.elapsed_time(e1) / launches)
        return statistics.median(per), min(per)

    def check(self, points=4096, which=0):
        """The output buffer of tensor set `which` as the timed launches left it, against the CPU oracle on a seeded
        sample of output elements (plus the first and last ones).  Returns the gated figure (max |gpu - ref| over the
        sample, normalised by the largest |ref| of the sample) and the conditioning-relative error per element
        (|gpu - ref| / (sum |in * filt| + |bias|), its maximum): the checker leg, outside every timed region."""
        import numpy as np

        import oracle
        from paper_1611_06945_amd import workloads as wl

        w, s, torch = self.w, self.w.shape, self.torch
        torch.cuda.synchronize()
        o = self.sets[which][3]
        if w.dtype == wl.BF16:
            host = wl.storage_to_f64(o.view(torch.int16).cpu().numpy().view(np.uint16), w.dtype)
        else:
            host = o.cpu().numpy().astype(np.float64)
        if self.out_nhwc:
            host = np.ascontiguousarray(np.transpose(host, (0, 3, 1, 2)))
        n_out = host.size
        rng = np.random.default_rng(424242)
        idx = np.unique(np.concatenate([np.arange(min(32, n_out)), n_out - 1 - np.arange(min(32, n_out)),
                                        rng.integers(0, n_out, points)])).astype(np.int64)
        x = wl.storage_to_f64(self.data["in"], w.dtype)
        f = wl.storage_to_f64(self.data["filt"], w.dtype)
        b = self.data["bias"].astype(np.float64)
        if self.pool:
            # a pooled element is the maximum of the 9 convolution outputs under its window: those from the oracle
            n_, k_, py, px = np.unravel_index(idx, host.shape)
            win = np.stack([np.ravel_multi_index((n_, k_, 2 * py + dy, 2 * px + dx), (s.N, s.K, s.OH, s.OW))
                            for dy in range(3) for dx in range(3)], axis=1).astype(np.int64)
            ref9 = oracle.conv_fwd_points(x, f, b, win.ravel(), stride=s.stride, pad=s.pad, relu=True).reshape(win.shape)
            mag9 = oracle.conv_fwd_points(np.abs(x), np.abs(f), np.abs(b), win.ravel(), stride=s.stride, pad=s.pad,
                                          relu=False).reshape(win.shape)
            ref, mag = ref9.max(axis=1), mag9.max(axis=1)
        else:
            ref = oracle.conv_fwd_points(x, f, b, idx, stride=s.stride, pad=s.pad, relu=True)
            mag = oracle.conv_fwd_points(np.abs(x), np.abs(f), np.abs(b), idx, stride=s.stride, pad=s.pad, relu=False)
        got = host.ravel()[idx]
        if not np.all(np.isfinite(got)):
            raise RuntimeError("%s via %s: output holds NaN/Inf (unwritten or overflowed elements)" % (w.name, self.variant))
        diff = np.abs(got - ref)
        err = float(diff.max() / max(float(np.abs(ref).max()), 1e-30))
        cond = float((diff / np.maximum(mag, 1e-30)).max())
        lim = TOL[wl.DTYPE_NAMES[w.dtype]]
        if err > lim:
            raise RuntimeError("%s via %s: max normalised error %.3g over the limit %g" % (w.name, self.variant, err, lim))
        return {"max_norm_err": float("%.3g" % err), "limit": lim, "max_cond_rel_err": float("%.3g" % cond),
                "points": int(idx.size)}


_cpu_cache = {}


def cpu_layer_baseline(w, one_thread=False, budget_s=0.6):
    """The oracle timed on this host's cores on one whole layer (a warm-up pass on one image, then full passes for about
    `budget_s` seconds, at least one); cached per shape -- the oracle computes in fp64 whatever the storage type."""
    import numpy as np

    import oracle
    from paper_1611_06945_amd import workloads as wl

    s = w.shape
    key = (tuple(s.in_shape()), tuple(s.filt_shape()), s.stride, s.pad, one_thread)
    if key in _cpu_cache:
        return _cpu_cache[key]
    data = w.generate()
    x = wl.storage_to_f64(data["in"], w.dtype)
    f = wl.storage_to_f64(data["filt"], w.dtype)
    b = data["bias"].astype(np.float64)
    full = oracle.threads()
    if one_thread:
        oracle.set_threads(1)
    try:
        oracle.conv_fwd(x[:1], f, b, stride=s.stride, pad=s.pad, relu=True)
        n, t0 = 0, time.perf_counter()
        while True:
            oracle.conv_fwd(x, f, b, stride=s.stride, pad=s.pad, relu=True)
            n += 1
            dt = time.perf_counter() - t0
            if dt >= budget_s or n >= 2000:
                break
        cores = oracle.threads()
    finally:
        oracle.set_threads(full)
    rep = {"ms": round(dt / n * 1e3, 4), "gflops": round(s.flops * n / dt / 1e9, 3), "cores": cores, "passes": n, "kind": "oracle"}
    _cpu_cache[key] = rep
    return rep


def cpu_model():
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def algorithmic_bytes(w, r):
    """Bytes the operation has to move: input + filters + bias + output once each; with the fused pool the output is the
    pooled tensor (the convolution's own output is never stored)."""
    from paper_1611_06945_amd import workloads as wl

    s, es = w.shape, wl.DTYPE_BYTES[w.dtype]
    if not r.pool:
        return s.algorithmic_bytes(w.dtype)
    return s.algorithmic_bytes(w.dtype) - (s.N * s.K * s.OH * s.OW - s.N * s.K * r.oh * r.ow) * es


def layer_report(w, launches=100, batches=5, rotate_mb=0, fmt="nchw", cpu=True, cpu_one_thread=False):
    from paper_1611_06945_amd import workloads as wl

    dt = wl.DTYPE_NAMES[w.dtype]
    r = Resident(w, fmt=fmt)
    abytes = algorithmic_bytes(w, r)
    variant = r.autotune()
    med_h, _ = r.time_batches(launches, batches, warmup=20)
    med, mn = r.time_device(launches, batches)
    chk = r.check()
    executed = executed_mfma_flops(variant, w.shape)
    rep = {
        "layer": w.name + ("" if fmt == "nchw" else "+" + fmt), "N": w.shape.N, "dtype": dt, "format": fmt, "variant": variant,
        "ms": round(med, 6), "ms_min": round(mn, 6), "ms_host_loop": round(med_h, 6),
        "gflops": round(w.shape.flops / (med * 1e-3) / 1e9, 1),
        # fraction of the MFMA peak the matrix units really sustain (never above 1); for a Winograd variant the rate by
        # the paper's FLOP convention (FLOPs of the direct definition) is the separate `effective_frac_direct_flops`
        "frac_mfma_peak": round(executed / (med * 1e-3) / (PEAK_TFLOPS[dt] * 1e12), 5),
        "hbm_gbs_algorithmic": round(abytes / (med * 1e-3) / 1e9, 1),
        "frac_hbm_peak": round(abytes / (med * 1e-3) / (PEAK_HBM_GBS * 1e9), 5),
        "flops": w.shape.flops, "algorithmic_bytes": abytes,
        "max_norm_err": chk["max_norm_err"], "max_cond_rel_err": chk["max_cond_rel_err"], "checked_points": chk["points"],
    }
    if executed != w.shape.flops:
        rep["effective_frac_direct_flops"] = round(w.shape.flops / (med * 1e-3) / (PEAK_TFLOPS[dt] * 1e12), 5)
    if r.convert_us:
        rep["convert_us"] = r.convert_us
    if rotate_mb:
        # enough distinct tensor sets to exceed the last-level cache, so the figure is an HBM figure
        copies = max(2, int(rotate_mb * 1e6 / abytes) + 1)
        rr = Resident(w, copies=copies, fmt=fmt)
        rr.autotune()
        med_r, _ = rr.time_batches(max(launches, copies), batches, warmup=copies)
        rr.check(which=copies - 1)
        rep["ms_rotated"] = round(med_r, 6)
        rep["frac_hbm_peak_rotated"] = round(abytes / (med_r * 1e-3) / (PEAK_HBM_GBS * 1e9), 5)
        rep["rotated_copies"] = copies
    if cpu:
        rep["cpu_baseline"] = cpu_layer_baseline(w)
        if cpu_one_thread:
            rep["cpu_baseline_1_thread"] = cpu_layer_baseline(w, one_thread=True)
    return rep


def stack_report(dtype, batch=20, reps=50):
    """The five-layer stack end to end (all operations enqueued back to back by one conv_run_ops call per pass, one
    synchronisation at the end):
    every layer in [N][C][H][W], and with the data format chosen per layer (channel-innermost where it pays)."""
    import torch

    from paper_1611_06945_amd import binding as B
    from paper_1611_06945_amd import workloads as wl
    from paper_1611_06945_amd.stack import ConvStack

    layers = wl.config5_layers(batch, dtype)
    shapes = [w.shape for w in layers]
    gen = [w.generate() for w in layers]
    tdt = {wl.F16: torch.float16, wl.BF16: torch.bfloat16}[dtype]

    def up(a):
        import numpy as np

        if dtype == wl.BF16:
            return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(a).cuda()

    x = up(gen[0]["in"])
    filts = [up(g["filt"]) for g in gen]
    biases = [torch.from_numpy(g["bias"]).cuda() for g in gen]
    flops = sum(s.flops for s in shapes)
    rep = {"dtype": wl.DTYPE_NAMES[dtype], "N": batch, "flops": flops}
    for tag, formats in (("nchw", None), ("selected", "auto")):
        st = ConvStack(shapes, dtype, pool_after=wl.STACK_POOL_AFTER, formats=formats)
        st.autotune(x, filts, biases)
        for _ in range(5):
            st.run(x, filts, biases)
        torch.cuda.synchronize()
        per = []
        for _ in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                st.run(x, filts, biases)
            e1.record()
            e1.synchronize()
            per.append(e0.elapsed_time(e1) / reps)
        ms = statistics.median(per)
        per = []
        for _ in range(3):   # the same chain issued with one Python call per operation, for comparison
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                st.run_stepwise(x, filts, biases)
            e1.record()
            e1.synchronize()
            per.append(e0.elapsed_time(e1) / reps)
        ms_step = statistics.median(per)
        rep[tag] = {"ms_call_per_operation": round(ms_step, 5), "formats": st.formats, "filter_formats": st.filt_formats, "pool_fused": st.fused, "ms": round(ms, 5),
                    "gflops": round(flops / (ms * 1e-3) / 1e9, 1),
                    "variants": [B.conv_variant_name(d, -1) for d in st.descs]}
        # the same chain recorded once into a HIP graph and replayed: one launch per pass instead of one per operation
        graph = st.capture(x, filts, biases)
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        per = []
        for _ in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                graph.replay()
            e1.record()
            e1.synchronize()
            per.append(e0.elapsed_time(e1) / reps)
        rep[tag]["graph_ms"] = round(statistics.median(per), 5)
        del graph
        if st.plan_times:
            rep[tag]["planned_us"] = round(st.plan_times["total_us"], 2)
        del st
    return rep


def cpu_baseline(w, budget_s=12.0):
    """The oracle as it stands, timed on this host's cores on the same workload (whole layer, repeated)."""
    import numpy as np

    import oracle
    from paper_1611_06945_amd import workloads as wl

    data = w.generate()
    x = wl.storage_to_f64(data["in"], w.dtype)
    f = wl.storage_to_f64(data["filt"], w.dtype)
    b = data["bias"].astype(np.float64)
    oracle.conv_fwd(x[:1], f, b, stride=w.shape.stride, pad=w.shape.pad, relu=True)  # load + thread pool warm-up
    n, t0 = 0, time.perf_counter()
    while True:
        oracle.conv_fwd(x, f, b, stride=w.shape.stride, pad=w.shape.pad, relu=True)
        n += 1
        dt = time.perf_counter() - t0
        if dt >= budget_s or n >= 1000:
            break
    return {"value": round(w.shape.flops * n / dt / 1e9, 3), "unit": "GFLOP/s", "cores": oracle.threads(),
            "kind": "oracle", "ms_per_step": round(dt / n * 1e3, 3), "cpu_model": cpu_model(),
            "sample": "%d full passes of %s (fp64 direct convolution, %.1f s)" % (n, w.name, dt)}


def sweep_appendix_a(batch, dtype, table_out=None, launches=100, batches=5):
    """The paper's whole benchmark set (Appendix A) through the autotuner: per operation the selected variant, its time
    and rates, and the comparison the paper draws between per-operation tuning and one variant for everything."""
    from paper_1611_06945_amd import binding as B
    from paper_1611_06945_amd import workloads as wl

    dt = wl.DTYPE_NAMES[dtype]
    ops, per_variant = [], {}
    for w in wl.appendix_a(batch, dtype):
        r = Resident(w)
        chosen = r.autotune()
        n = B.conv_variant_count(r.desc)
        times = {B.conv_variant_name(r.desc, i): B.conv_variant_time_us(r.desc, i) for i in range(n)}
        med_h, _ = r.time_batches(launches, batches, warmup=20)
        med, mn = r.time_device(launches, batches)
        abytes = w.shape.algorithmic_bytes(w.dtype)
        t_mfma = w.shape.flops / (PEAK_TFLOPS[dt] * 1e12)
        t_hbm = abytes / (PEAK_HBM_GBS * 1e9)
        ops.append({"op": w.name, "paper_row": w.paper_row, "flops": w.shape.flops, "algorithmic_bytes": abytes,
                    "variant": chosen, "ms": round(med, 6), "ms_min": round(mn, 6), "ms_host_loop": round(med_h, 6),
                    "tuner_us": round(times[chosen], 3),
                    "gflops": round(w.shape.flops / (med * 1e-3) / 1e9, 1),
                    "bound": "mfma" if t_mfma >= t_hbm else "hbm",
                    "frac_roofline": round(max(t_mfma, t_hbm) / (med * 1e-3), 5),
                    "n_variants": n})
        executed = executed_mfma_flops(chosen, w.shape)
        if ops[-1]["bound"] == "mfma" and executed != w.shape.flops:
            # a Winograd variant: the fraction of the MFMA peak counts the FLOPs the matrix units execute (never above 1);
            # the rate by the direct definition's FLOP count stays in `gflops` and `effective_frac_direct_flops`
            ops[-1]["effective_frac_direct_flops"] = ops[-1]["frac_roofline"]
            ops[-1]["frac_roofline"] = round(executed / (PEAK_TFLOPS[dt] * 1e12) / (med * 1e-3), 5)
        if ops[-1]["bound"] == "hbm":
            # stream-bound operation: repeat over enough distinct tensor sets to defeat the 256 MB last-level cache
            copies = max(2, int(600e6 / abytes) + 1)
            rr = Resident(w, copies=copies)
            rr.autotune()
            med_r, _ = rr.time_batches(max(50, 2 * copies), 3, warmup=copies)
            ops[-1]["ms_rotated"] = round(med_r, 6)
            ops[-1]["frac_roofline_rotated"] = round(t_hbm / (med_r * 1e-3), 5)
            ops[-1]["rotated_copies"] = copies
            del rr
        for name, t in times.items():
            per_variant.setdefault(name, {})[w.name] = t
        log("%-46s %-40s %8.4f ms %9.1f GFLOP/s  roofline %.3f (%s)" % (
            w.name, chosen, med, ops[-1]["gflops"], ops[-1]["frac_roofline"], ops[-1]["bound"]))
        del r
    # one variant for every operation: the variant valid on all of them with the smallest summed time
    everywhere = {name: sum(t.values()) for name, t in per_variant.items() if len(t) == len(ops)}
    single = min(everywhere, key=everywhere.get) if everywhere else None
    for o in ops:
        o["single_variant_us"] = round(per_variant[single][o["op"]], 3) if single else None
        o["tuning_gain"] = round(o["single_variant_us"] / o["tuner_us"], 3) if single else None
    tot_flops = sum(o["flops"] for o in ops)
    tot_ms = sum(o["ms"] for o in ops)
    summary = {
        "workload": "appendix_a_n%d_%s" % (batch, dt), "ops": len(ops), "total_flops": tot_flops,
        "total_ms": round(tot_ms, 5), "gflops": round(tot_flops / (tot_ms * 1e-3) / 1e9, 1),
        "single_variant": single,
        "single_variant_total_us": round(everywhere[single], 2) if single else None,
        "autotuned_total_us": round(sum(o["tuner_us"] for o in ops), 2),
        "variants_valid_everywhere": len(everywhere),
    }
    if table_out:
        with open(table_out, "w") as fh:
            fh.write("command (repo root, one MI355X): python3 bench.py --sweep appendix_a --sweep-batch %d --sweep-dtype %s --table-out %s\n\n"
                     % (batch, dt, table_out))
            fh.write("ms: per launch, device events around batches of launches issued by the library (conv_time_us; median); "
                     "tuner us: the same variant as timed by the autotuner; one-variant us: the single variant valid on "
                     "every operation with the smallest total, timed the same way; gain = one-variant / tuner.  GFLOP and "
                     "GFLOP/s count the FLOPs of the direct definition; for a Winograd variant (wino_*) the fraction of the roofline "
                     "counts the FLOPs its matrix instructions execute (2.25x fewer).\n\n")
            fh.write("| # | operation (KSZ,S,OC, in -> out) | GFLOP | variant | ms | tuner us | GFLOP/s | bound | frac of roofline | one-variant us | gain |\n")
            fh.write("|---|---|---|---|---|---|---|---|---|---|---|\n")
            for i, o in enumerate(ops):
                fh.write("| %d | %s | %.3f | %s | %.4f | %.2f | %.0f | %s | %.3f | %s | %s |\n" % (
                    i, o["paper_row"], o["flops"] / 1e9, o["variant"], o["ms"], o["tuner_us"], o["gflops"], o["bound"],
                    o["frac_roofline"], o["single_variant_us"], o["tuning_gain"]))
            rot = [o for o in ops if "ms_rotated" in o]
            if rot:
                fh.write("\nStream-bound operations repeated over distinct tensor sets larger than the last-level cache "
                         "(host loop): " + "; ".join("#%d %.4f ms = %.3f of the HBM roofline (%d sets)" % (
                             ops.index(o), o["ms_rotated"], o["frac_roofline_rotated"], o["rotated_copies"]) for o in rot) + "\n")
            fh.write("\n" + json.dumps(summary) + "\n")
    return summary, ops


def stored_traffic(kernel_key):
    """HBM bytes per launch measured offline with rocprofv3 --pmc (see profiles/).  A variant without a record gets an
    explicit text instead of a number, so that a missing measurement cannot pass for one."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as fh:
            rec = json.load(fh).get(kernel_key)
    except (OSError, ValueError):
        rec = None
    if rec is None or rec.get("total_bytes") is None:
        log("warning: no FETCH_SIZE/WRITE_SIZE record for %s in profiles/hbm_traffic.json" % kernel_key)
        return "not recorded for %s" % kernel_key
    return rec["total_bytes"]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", default="cfg4_mid3x3_n20_f32")
    ap.add_argument("--variant", help="run the headline workload on this variant instead of the autotuned one "
                                      "(for profiling one kernel; the figure is then not the headline)")
    ap.add_argument("--format", choices=["nchw", "nhwc", "nhwc_packed", "nchw_pool"], default="nchw",
                    help="tensor formats of the workload (16-bit layers only for the channel-innermost ones); anything but "
                         "nchw is for profiling one kernel: the headline stays on the plain contract")
    ap.add_argument("--probe", action="store_true", help="print the device microbenchmarks (MFMA issue rate by occupancy and "
                                                         "interleaved vector-ALU work, copy bandwidth) and exit")
    ap.add_argument("--no-layers", action="store_true", help="skip the per-layer table")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--sweep", choices=["appendix_a"], help="time the paper's whole benchmark set instead of one workload")
    ap.add_argument("--sweep-batch", type=int, default=5)
    ap.add_argument("--sweep-dtype", choices=["f32", "f16", "bf16"], default="f32")
    ap.add_argument("--table-out", help="with --sweep: also write the per-operation table (markdown) to this file")
    a = ap.parse_args()
    if a.gpus != 1:
        log("bench.py: this build runs on ONE GPU (the paper's method is single-device inference); --gpus %d is not "
            "supported." % a.gpus)
        sys.exit(2)

    import torch

    from paper_1611_06945_amd import binding as B
    from paper_1611_06945_amd import workloads as wl

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(3)
    B.lib()  # fail loudly if the HIP library is not built
    torch.cuda.set_device(0)
    log("device:", torch.cuda.get_device_name(0))

    if a.probe:
        scratch = torch.zeros(64, device="cuda")
        rows = []
        for code, name in ((wl.F16, "f16"), (wl.BF16, "bf16"), (wl.F32, "f32")):
            for block in (32, 16):
                for wps in (1, 2, 4):
                    for nv in (0, 2, 4, 8):
                        tf, ns = B.conv_probe_mfma_mix(code, block, wps, nv, scratch)
                        rows.append({"dtype": name, "block": block, "waves_per_simd": wps, "valu_per_mfma": nv,
                                     "tflops": round(tf, 1), "ns_per_mfma": round(ns, 2)})
                        log("mfma %-4s %2dx%-2d  %d waves/SIMD  %d VALU per MFMA: %8.1f TFLOP/s  %6.2f ns per MFMA and SIMD" % (
                            name, block, block, wps, nv, tf, ns))
        for code, name in ((wl.F16, "f16"), (wl.BF16, "bf16")):
            for wps in (1, 2, 4):
                tf, ns = B.conv_probe_mfma_mix(code, 32, wps, 0, scratch, distinct_operands=True)
                rows.append({"dtype": name, "block": 32, "waves_per_simd": wps, "valu_per_mfma": 0, "distinct_operands": True,
                             "tflops": round(tf, 1), "ns_per_mfma": round(ns, 2)})
                log("mfma %-4s 32x32  %d waves/SIMD  operand registers of its own per MFMA: %8.1f TFLOP/s  %6.2f ns per MFMA and SIMD" % (
                    name, wps, tf, ns))
        big = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        big2 = torch.empty_like(big)
        copy = round(B.conv_probe_stream_bandwidth(big, big2, big.numel()), 1)
        log("1 GiB device-to-device copy: %.1f GB/s (read + written bytes)" % copy)
        print(json.dumps({"probe": "mfma_mix", "rows": rows, "stream_copy_gbs": copy}), flush=True)
        return

    if a.sweep:
        code = {"f32": wl.F32, "f16": wl.F16, "bf16": wl.BF16}[a.sweep_dtype]
        summary, ops = sweep_appendix_a(a.sweep_batch, code, a.table_out)
        log("sweep:", summary)
        print(json.dumps({
            "metric": "conv_fwd_gflops", "value": summary["gflops"], "unit": "GFLOP/s", "n_gpus": 1,
            "steps": len(ops), "warmup": 0, "ms_per_step": summary["total_ms"], "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": a.sweep_dtype, "data": "synthetic",
            "config": {"workload": summary["workload"], "fused": "bias+relu"}, "sweep": summary, "ops": ops}), flush=True)
        return

    table = {w.name: w for w in all_workloads()}
    for code in (wl.F32, wl.F16, wl.BF16):   # the rows of the paper's Appendix A at batch 5, for profiling single operations
        table.update({w.name: w for w in wl.appendix_a(5, code)})
    if a.workload not in table:
        log("unknown workload %r; choose from %s" % (a.workload, sorted(table)))
        sys.exit(2)
    w = table[a.workload]
    dt = wl.DTYPE_NAMES[w.dtype]

    # ---- headline: exactly `steps` timed steps after `warmup` untimed ones --------------------------------
    r = Resident(w, fmt=a.format)
    if a.variant:
        # profiling one kernel: no autotuning pass, so that a trace of this run holds this variant's launches only
        names = [B.conv_variant_name(r.desc, i) for i in range(B.conv_variant_count(r.desc))]
        if a.variant not in names:
            log("variant %r is not valid for %s; choose from %s" % (a.variant, w.name, names))
            sys.exit(2)
        B.conv_force_variant(r.desc, names.index(a.variant))
        variant = r.variant = a.variant
    else:
        variant = r.autotune()
    log("headline %s -> %s%s" % (w.name, variant, " (forced)" if a.variant else ""))
    for _ in range(a.warmup):
        r.step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(a.steps):
        r.step()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ev_ms = e0.elapsed_time(e1)
    ms_per_step = wall_ms / a.steps
    kern_ms = ev_ms / a.steps  # device-side average per launch over the timed region
    gflops = w.shape.flops / (ms_per_step * 1e-3) / 1e9
    check = r.check()          # the output the timed launches left behind, against the oracle (raises over the limit)
    log("checked %d outputs of the timed run against the oracle: max normalised error %.3g (limit %g), conditioning-relative %.3g" % (
        check["points"], check["max_norm_err"], check["limit"], check["max_cond_rel_err"]))

    head_bytes = algorithmic_bytes(w, r)
    mfma_bound = w.shape.flops / (PEAK_TFLOPS[dt] * 1e12) >= head_bytes / (PEAK_HBM_GBS * 1e9)
    executed = executed_mfma_flops(variant, w.shape)
    if mfma_bound:
        # `achieved` / `frac`: what the matrix units sustain (FLOPs they execute / time), which cannot exceed the peak.  For
        # a Winograd variant that is 2.25x fewer FLOPs than the direct definition's; the rate by the paper's FLOP
        # convention (how it also rates the vendor library's Winograd kernels) is `effective_*_direct_flops`.
        ach = executed / (kern_ms * 1e-3) / 1e12
        roof = {"bound": "mfma", "achieved": round(ach, 3), "peak": PEAK_TFLOPS[dt], "unit": "TFLOP/s",
                "frac": round(ach / PEAK_TFLOPS[dt], 5), "flops_counted": "executed by the matrix units",
                "mfma_flops_executed": executed, "algorithmic_flops": w.shape.flops,
                "effective_tflops_direct_flops": round(w.shape.flops / (kern_ms * 1e-3) / 1e12, 3),
                "effective_frac_direct_flops": round(w.shape.flops / (kern_ms * 1e-3) / 1e12 / PEAK_TFLOPS[dt], 5)}
    else:
        ach = head_bytes / (kern_ms * 1e-3) / 1e9
        roof = {"bound": "hbm", "achieved": round(ach, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": round(ach / PEAK_HBM_GBS, 5)}
    # measured ceilings of this very device, next to the published ones
    scratch = torch.zeros(64, device="cuda")
    big = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    big2 = torch.empty_like(big)
    measured = {"mfma_tflops": {}, "stream_copy_gbs": round(B.conv_probe_stream_bandwidth(big, big2, big.numel()), 1),
                "note": "register-only MFMA issue loop (best block shape) and 1 GiB device-to-device copy (read+write bytes)"}
    for code, name in ((wl.F32, "f32"), (wl.F16, "f16"), (wl.BF16, "bf16")):
        measured["mfma_tflops"][name] = round(max(B.conv_probe_mfma_peak(code, 32, scratch), B.conv_probe_mfma_peak(code, 16, scratch)), 1)
    del big, big2
    roof["frac_of_measured"] = round(ach / (measured["mfma_tflops"][dt] if mfma_bound else measured["stream_copy_gbs"]), 5)
    roof["traffic"] = stored_traffic("%s|%s" % (w.name, variant))
    roof["kernel"] = variant
    roof["kernel_ms"] = round(kern_ms, 6)
    if variant.startswith("wino_") and not a.variant:
        # next to the fastest direct variant the tuner measured, and the same layer with pre-transformed filters
        sh = w.shape
        fused = variant.endswith("_ff")
        roof["algorithm"] = ("winograd F(2x2,3x3): one kernel per launch (filter, input and output transforms around the MFMA planes)"
                             if fused else "winograd F(2x2,3x3): filter transform kernel + fused product kernel per launch")
        n = B.conv_variant_count(r.desc)
        direct = [(B.conv_variant_time_us(r.desc, i), B.conv_variant_name(r.desc, i)) for i in range(n)]
        direct = [x for x in direct if not x[1].startswith("wino_") and x[0] > 0]
        # the same layer with the filters handed over in the Winograd domain (the transform is then a conversion done
        # once, ahead of time, as the paper does for constant weights): an extra figure, never the headline value
        pre = B.desc_of(sh, w.dtype, relu=True, filt_winograd=True)
        if B.conv_variant_count(pre) > 0:
            x, f, b, o = r.sets[0]
            u = torch.empty(B.conv_transformed_filter_bytes(pre), dtype=torch.uint8, device="cuda")
            B.conv_transform_filters(pre, f, u)
            B.conv_autotune(pre, x, u, b, o, None, 0)
            us = min(B.conv_time_us(pre, x, u, b, o, None, 0, launches=200) for _ in range(3))
            pre_variant = B.conv_variant_name(pre, -1)
            roof["pretransformed_filters"] = {"variant": pre_variant, "us": round(us, 2),
                                              "tflops": round(sh.flops / (us * 1e-6) / 1e12, 2),
                                              "frac": round(executed_mfma_flops(pre_variant, sh) / (us * 1e-6) / 1e12 / PEAK_TFLOPS[dt], 5),
                                              "effective_frac_direct_flops": round(sh.flops / (us * 1e-6) / 1e12 / PEAK_TFLOPS[dt], 5)}
        if direct:
            t_us, nm = min(direct)
            roof["best_direct"] = {"variant": nm, "tuner_us": round(t_us, 2),
                                   "frac": round(sh.flops / (t_us * 1e-6) / 1e12 / PEAK_TFLOPS[dt], 5)}

    out = {
        "metric": "conv_fwd_gflops", "value": round(gflops, 1), "unit": "GFLOP/s", "n_gpus": 1,
        "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(ms_per_step, 6), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": dt, "data": "synthetic",
        "config": {"workload": w.name, "N": w.shape.N, "C": w.shape.C, "H": w.shape.H, "W": w.shape.W,
                   "K": w.shape.K, "R": w.shape.R, "S": w.shape.S, "stride": w.shape.stride, "pad": w.shape.pad,
                   "fused": "bias+relu", "format": a.format, "variant": variant, "paper_row": w.paper_row},
        "variant": variant, "max_norm_err": check["max_norm_err"], "max_cond_rel_err": check["max_cond_rel_err"],
        "checked_points": check["points"], "tolerance": check["limit"],
        "roofline": roof,
        "measured_peaks": measured,
    }

    if not a.no_layers:
        layers = []
        entries = [(lw, "nchw") for lw in all_workloads()]
        # the 16-bit 3x3 / 5x5 layers again on channel-innermost tensors with the filters in MFMA operand order (explicit
        # ahead-of-time conversions, timed separately in `convert_us`): the format the stack planner selects for them
        entries += [(lw, "nhwc_packed") for lw in all_workloads()
                    if lw.dtype == wl.F16 and (lw.name.startswith("cfg4") or lw.name[:7] in ("cfg5_L2", "cfg5_L3", "cfg5_L4", "cfg5_L5"))]
        # the stack's first layer with its 3x3 stride-2 pool computed by the convolution kernel (pooled output)
        entries += [(lw, "nchw_pool") for lw in all_workloads() if lw.dtype == wl.F16 and lw.name.startswith("cfg5_L1")]
        for lw, fmt in entries:
            hbmish = lw.name.startswith("cfg2") or lw.name.startswith("cfg5_L1") or (lw.shape.N == 1 and lw.dtype != wl.F32)
            small = lw.name.startswith(("cfg1", "cfg2")) or (lw.name.startswith("cfg4") and lw.shape.N == 1)
            rep = layer_report(lw, rotate_mb=300 if hbmish else 0, fmt=fmt, cpu=not a.no_cpu, cpu_one_thread=small)
            layers.append(rep)
            log("%-34s %-44s %9.4f ms %10.1f GFLOP/s  mfma %.3f  hbm %.3f  err %.2g%s" % (
                rep["layer"], rep["variant"], rep["ms"], rep["gflops"], rep["frac_mfma_peak"], rep["frac_hbm_peak"],
                rep["max_norm_err"], "  cpu %.1f GFLOP/s" % rep["cpu_baseline"]["gflops"] if "cpu_baseline" in rep else ""))
        out["layers"] = layers
        out["stack"] = stack_report(wl.F16)
        log("stack f16: all-NCHW %.4f ms (HIP graph %.4f), formats selected %s filters %s pools fused %s %.4f ms (HIP graph %.4f)" % (
            out["stack"]["nchw"]["ms"], out["stack"]["nchw"]["graph_ms"], out["stack"]["selected"]["formats"],
            out["stack"]["selected"]["filter_formats"], out["stack"]["selected"]["pool_fused"], out["stack"]["selected"]["ms"],
            out["stack"]["selected"]["graph_ms"]))

    if not a.no_cpu:
        out["cpu_baseline"] = cpu_baseline(w)
        out["cpu_model"] = cpu_model()
        log("cpu oracle:", out["cpu_baseline"])

    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
