#!/usr/bin/env python3
"""Forward-convolution benchmark on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-layers] [--no-cpu]

A step is one call of the fused convolution (conv_fwd_ws through the C ABI: filter-tile and patch-tile staging,
MFMA main loop, fused bias+ReLU store; plus the fixed-order reduce when a split variant is selected) on one
batch of seeded synthetic input that is already resident in device memory.  The variant is chosen by the
library's autotuner before timing starts.  The headline workload is the mid-network 3x3 layer of the batch
sweep at batch 20 in fp32 (the paper's arithmetic); `layers` in the JSON line reports every benchmark layer at
batch 1/5/20 and every storage type: ms, GFLOP/s and the fraction of the MFMA and HBM rooflines.

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


class Resident:
    """A workload with its tensors in device memory (optionally several rotating copies)."""

    def __init__(self, w, copies=1):
        import torch

        from paper_1611_06945_amd import binding as B
        from paper_1611_06945_amd import workloads as wl

        self.w, self.B, self.torch = w, B, torch
        self.desc = B.desc_of(w.shape, w.dtype, relu=True)
        data = w.generate()
        tdt = {wl.F32: torch.float32, wl.F16: torch.float16, wl.BF16: torch.bfloat16}[w.dtype]

        def up(a):
            if w.dtype == wl.BF16:
                import numpy as np

                return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
            return torch.from_numpy(a).cuda()

        self.sets = []
        for _ in range(copies):
            self.sets.append((up(data["in"]).clone(), up(data["filt"]).clone(), torch.from_numpy(data["bias"]).cuda(),
                              torch.empty(w.shape.out_shape(), dtype=tdt, device="cuda")))
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


def layer_report(w, launches=100, batches=5, rotate_mb=0):
    from paper_1611_06945_amd import workloads as wl

    dt = wl.DTYPE_NAMES[w.dtype]
    abytes = w.shape.algorithmic_bytes(w.dtype)
    r = Resident(w)
    variant = r.autotune()
    med_h, _ = r.time_batches(launches, batches, warmup=20)
    med, mn = r.time_device(launches, batches)
    rep = {
        "layer": w.name, "N": w.shape.N, "dtype": dt, "variant": variant,
        "ms": round(med, 6), "ms_min": round(mn, 6), "ms_host_loop": round(med_h, 6),
        "gflops": round(w.shape.flops / (med * 1e-3) / 1e9, 1),
        "frac_mfma_peak": round(w.shape.flops / (med * 1e-3) / (PEAK_TFLOPS[dt] * 1e12), 5),
        "hbm_gbs_algorithmic": round(abytes / (med * 1e-3) / 1e9, 1),
        "frac_hbm_peak": round(abytes / (med * 1e-3) / (PEAK_HBM_GBS * 1e9), 5),
        "flops": w.shape.flops, "algorithmic_bytes": abytes,
    }
    if rotate_mb:
        # enough distinct tensor sets to exceed the last-level cache, so the figure is an HBM figure
        copies = max(2, int(rotate_mb * 1e6 / abytes) + 1)
        rr = Resident(w, copies=copies)
        rr.autotune()
        med_r, _ = rr.time_batches(max(launches, copies), batches, warmup=copies)
        rep["ms_rotated"] = round(med_r, 6)
        rep["frac_hbm_peak_rotated"] = round(abytes / (med_r * 1e-3) / (PEAK_HBM_GBS * 1e9), 5)
        rep["rotated_copies"] = copies
    return rep


def stack_report(dtype, batch=20, reps=50):
    """The five-layer stack end to end (all operations enqueued back to back, one synchronisation at the end):
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
        rep[tag] = {"formats": st.formats, "pool_fused": st.fused, "ms": round(ms, 5),
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
            "kind": "oracle", "ms_per_step": round(dt / n * 1e3, 3),
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
            fh.write("ms: per launch, device events around batches of launches issued by the library (conv_time_us; median); "
                     "tuner us: the same variant as timed by the autotuner; one-variant us: the single variant valid on "
                     "every operation with the smallest total, timed the same way; gain = one-variant / tuner.\n\n")
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
    """HBM bytes per launch measured offline with rocprofv3 --pmc (see profiles/); None if not recorded."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as fh:
            rec = json.load(fh).get(kernel_key)
            return None if rec is None else rec.get("total_bytes")
    except (OSError, ValueError):
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", default="cfg4_mid3x3_n20_f32")
    ap.add_argument("--variant", help="run the headline workload on this variant instead of the autotuned one "
                                      "(for profiling one kernel; the figure is then not the headline)")
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
    if a.workload not in table:
        log("unknown workload %r; choose from %s" % (a.workload, sorted(table)))
        sys.exit(2)
    w = table[a.workload]
    dt = wl.DTYPE_NAMES[w.dtype]

    # ---- headline: exactly `steps` timed steps after `warmup` untimed ones --------------------------------
    r = Resident(w)
    variant = r.autotune()
    if a.variant:
        names = [B.conv_variant_name(r.desc, i) for i in range(B.conv_variant_count(r.desc))]
        if a.variant not in names:
            log("variant %r is not valid for %s; choose from %s" % (a.variant, w.name, names))
            sys.exit(2)
        B.conv_force_variant(r.desc, names.index(a.variant))
        variant = r.variant = a.variant
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

    mfma_bound = w.shape.flops / (PEAK_TFLOPS[dt] * 1e12) >= w.shape.algorithmic_bytes(w.dtype) / (PEAK_HBM_GBS * 1e9)
    if mfma_bound:
        ach = w.shape.flops / (kern_ms * 1e-3) / 1e12
        roof = {"bound": "mfma", "achieved": round(ach, 3), "peak": PEAK_TFLOPS[dt], "unit": "TFLOP/s",
                "frac": round(ach / PEAK_TFLOPS[dt], 5)}
    else:
        ach = w.shape.algorithmic_bytes(w.dtype) / (kern_ms * 1e-3) / 1e9
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
    if variant.startswith("wino_"):
        # `achieved` above counts the FLOPs of the direct definition (the paper's per-operation FLOP count, which is how it
        # also rates the vendor library's Winograd kernels); the MFMA units execute 2.25x fewer multiplications, on tiles
        # padded to the workgroup shape.  Both views are reported, next to the fastest direct variant the tuner measured.
        import re
        sh = w.shape
        tiles = sh.N * ((sh.OH + 1) // 2) * ((sh.OW + 1) // 2)

        def executed_flops(name):
            m = re.match(r"wino_f32_M(\d+)T(\d+)_", name)
            tm, tt = int(m.group(1)), int(m.group(2))
            return 2.0 * 16 * (-(-sh.K // tm) * tm) * (-(-tiles // tt) * tt) * sh.C

        executed = executed_flops(variant)
        fused = variant.endswith("_ff")
        roof["algorithm"] = ("winograd F(2x2,3x3): one kernel per launch (filter, input and output transforms around the MFMA planes)"
                             if fused else "winograd F(2x2,3x3): filter transform kernel + fused product kernel per launch")
        roof["mfma_flops_executed"] = executed
        roof["frac_executed"] = round(executed / (kern_ms * 1e-3) / 1e12 / PEAK_TFLOPS[dt], 5)
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
                                              "frac": round(sh.flops / (us * 1e-6) / 1e12 / PEAK_TFLOPS[dt], 5),
                                              "frac_executed": round(executed_flops(pre_variant) / (us * 1e-6) / 1e12 / PEAK_TFLOPS[dt], 5)}
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
                   "fused": "bias+relu", "variant": variant, "paper_row": w.paper_row},
        "roofline": roof,
        "measured_peaks": measured,
    }

    if not a.no_layers:
        layers = []
        for lw in all_workloads():
            hbmish = lw.name.startswith("cfg2") or lw.name.startswith("cfg5_L1") or (lw.shape.N == 1 and lw.dtype != wl.F32)
            rep = layer_report(lw, rotate_mb=300 if hbmish else 0)
            layers.append(rep)
            log("%-26s %-44s %9.4f ms %10.1f GFLOP/s  mfma %.3f  hbm %.3f" % (
                rep["layer"], rep["variant"], rep["ms"], rep["gflops"], rep["frac_mfma_peak"], rep["frac_hbm_peak"]))
        out["layers"] = layers
        out["stack"] = stack_report(wl.F16)
        log("stack f16: all-NCHW %.4f ms (HIP graph %.4f), formats selected %s pools fused %s %.4f ms (HIP graph %.4f)" % (
            out["stack"]["nchw"]["ms"], out["stack"]["nchw"]["graph_ms"], out["stack"]["selected"]["formats"],
            out["stack"]["selected"]["pool_fused"], out["stack"]["selected"]["ms"], out["stack"]["selected"]["graph_ms"]))

    if not a.no_cpu:
        out["cpu_baseline"] = cpu_baseline(w)
        log("cpu oracle:", out["cpu_baseline"])

    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
