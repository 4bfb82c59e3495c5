"""GPU parity at the full benchmark sizes, in the launch configuration the bench times
(autotuned selection, workspace available), every output element against the CPU oracle."""
import numpy as np
import pytest

import oracle
from paper_1611_06945_amd import binding as B
from paper_1611_06945_amd import workloads as wl
from paper_1611_06945_amd.stack import ConvStack

from gpu_util import TOL, DeviceCase, empty_out, to_device, to_host_f64, to_host_stored, torch_mod

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def check_workload(w, autotune=True):
    case = DeviceCase(w.shape, w.dtype, w.generate(), relu=True, use_bias=True)
    say("  %s: heuristic picks %s / %s" % (w.name, B.conv_variant_name(case.desc, -1), B.conv_variant_name(case.desc, -2)))
    e1 = case.error(case.run(with_ws=True))
    e2 = case.error(case.run(with_ws=False))
    assert e1 <= TOL[w.dtype] and e2 <= TOL[w.dtype], (w.name, e1, e2)
    if autotune:
        ws = case.workspace()
        out = empty_out(w.shape.out_shape(), w.dtype)
        B.conv_autotune(case.desc, case.d_in, case.d_filt, case.d_bias, out, ws, ws.numel())
        say("  %s: autotuned picks %s / %s" % (w.name, B.conv_variant_name(case.desc, -1), B.conv_variant_name(case.desc, -2)))
        e3 = case.error(case.run(with_ws=True))
        e4 = case.error(case.run(with_ws=False))
        assert e3 <= TOL[w.dtype] and e4 <= TOL[w.dtype], (w.name, e3, e4)
        say("  %s: max normalised error %.3g (limit %.1g)" % (w.name, max(e1, e2, e3, e4), TOL[w.dtype]))
    return case


def test_config1_toy_layer():
    check_workload(wl.config1())


def test_config2_pointwise():
    case = check_workload(wl.config2())
    assert any(n.startswith("pw_") for n in case.variant_names())


def test_config3_first_layer():
    check_workload(wl.config3())


@pytest.mark.parametrize("dtype", [wl.F32, wl.F16, wl.BF16])
@pytest.mark.parametrize("batch", [1, 5, 20])
def test_config4_mid_network_batch_sweep(batch, dtype):
    check_workload(wl.config4(batch, dtype))


@pytest.mark.parametrize("dtype", [wl.F16, wl.BF16])
def test_config5_stack(dtype):
    torch = torch_mod()
    layers = wl.config5_layers(20, dtype)
    shapes = [w.shape for w in layers]
    stack = ConvStack(shapes, dtype, pool_after=wl.STACK_POOL_AFTER)
    x_host = layers[0].generate()["in"]
    gen = [w.generate() for w in layers]
    filts_host = [g["filt"] for g in gen]
    bias_host = [g["bias"] for g in gen]
    x = to_device(x_host, dtype)
    filts = [to_device(f, dtype) for f in filts_host]
    biases = [to_device(b, wl.F32) for b in bias_host]
    stack.autotune(x, filts, biases)
    for d in stack.descs:
        say("  stack layer -> %s" % B.conv_variant_name(d, -1))
    y = stack.run(x, filts, biases)
    torch.cuda.synchronize()

    # (i) per layer: the oracle is fed the GPU's own stored input of that layer, so each kernel is judged alone
    cur_host = x_host
    ref_chain = wl.storage_to_f64(x_host, dtype)  # (ii) the oracle's own chain, rounded to storage between layers
    for i, s in enumerate(shapes):
        ref = oracle.conv_fwd(wl.storage_to_f64(cur_host, dtype), wl.storage_to_f64(filts_host[i], dtype),
                              bias_host[i].astype(np.float64), stride=s.stride, pad=s.pad, relu=True)
        got = to_host_f64(stack.conv_out[i], dtype)
        assert np.all(np.isfinite(got))
        err = oracle.max_normalised_error(got, ref)
        say("  layer %d per-layer error %.3g" % (i + 1, err))
        assert err <= TOL[dtype], (i + 1, err)
        chain = oracle.conv_fwd(ref_chain, wl.storage_to_f64(filts_host[i], dtype), bias_host[i].astype(np.float64),
                                stride=s.stride, pad=s.pad, relu=True)
        if stack.pool_out[i] is not None:
            pref = oracle.maxpool_fwd(got, win=3, stride=2)
            pgot = to_host_f64(stack.pool_out[i], dtype)
            assert np.array_equal(pgot, pref), "max-pool after layer %d" % (i + 1)
            chain = oracle.maxpool_fwd(chain, win=3, stride=2)
        cur_host = to_host_stored(stack.layer_output(i), dtype)
        ref_chain = wl.storage_to_f64(wl.to_storage(chain.astype(np.float32), dtype), dtype)
    e2e = oracle.max_normalised_error(to_host_f64(y, dtype), ref_chain)
    say("  end-to-end error vs the oracle's own chain: %.3g" % e2e)
    assert e2e <= 10 * TOL[dtype]


def _to_nchw(t, layout, dtype):
    """Logical [N][K][OH][OW] float64 view of a stack buffer stored in `layout`."""
    host = to_host_f64(t, dtype)
    if layout == "nhwc":
        n, k, h, w = host.shape
        host = np.ascontiguousarray(np.transpose(host.reshape(n, h, w, k), (0, 3, 1, 2)))
    return host


def _check_stack_against_oracle(stack, shapes, gen, dtype, y):
    """Every layer of a finished run against the oracle, each judged on the GPU's own stored input."""
    cur = wl.storage_to_f64(gen[0]["in"], dtype)
    for i, s in enumerate(shapes):
        ref = oracle.conv_fwd(cur, wl.storage_to_f64(gen[i]["filt"], dtype), gen[i]["bias"].astype(np.float64),
                              stride=s.stride, pad=s.pad, relu=True)
        handed = _to_nchw(stack.layer_output(i), stack.output_layout(i), dtype)
        if stack.fused[i]:  # the convolution's own output is never stored: compare the pooled tensor
            assert stack.conv_out[i] is None
            err = oracle.max_normalised_error(handed, oracle.maxpool_fwd(ref, win=3, stride=2))
            say("  layer %d + pool (%s, %s) error %.3g" % (i + 1, stack.formats[i], B.conv_variant_name(stack.descs[i], -1), err))
            assert np.all(np.isfinite(handed)) and err <= TOL[dtype], (i + 1, err)
            cur = handed
            continue
        got = _to_nchw(stack.conv_out[i], stack.conv_layout[i], dtype)
        assert np.all(np.isfinite(got))
        err = oracle.max_normalised_error(got, ref)
        say("  layer %d (%s, %s) error %.3g" % (i + 1, stack.formats[i], B.conv_variant_name(stack.descs[i], -1), err))
        assert err <= TOL[dtype], (i + 1, err)
        if stack.pool_out[i] is not None:
            assert np.array_equal(handed, oracle.maxpool_fwd(got, win=3, stride=2)), "max-pool after layer %d" % (i + 1)
        else:
            assert np.array_equal(handed, got), "conversion after layer %d" % (i + 1)
        cur = handed  # the next layer is judged on the GPU's own stored input
    assert stack.output_layout(len(shapes) - 1) == "nchw"
    assert np.array_equal(to_host_f64(y, dtype), cur)


def _stack_on_device(dtype, batch, **kw):
    layers = wl.config5_layers(batch, dtype)
    shapes = [w.shape for w in layers]
    stack = ConvStack(shapes, dtype, pool_after=wl.STACK_POOL_AFTER, **kw)
    gen = [w.generate() for w in layers]
    x = to_device(gen[0]["in"], dtype)
    filts = [to_device(g["filt"], dtype) for g in gen]
    biases = [to_device(g["bias"], wl.F32) for g in gen]
    return stack, shapes, gen, x, filts, biases


@pytest.mark.parametrize("formats", [["nchw", "nhwc", "nchw", "nhwc", "nhwc"],
                                     ["nchw", "nhwc_packed", "nhwc_packed", "nhwc", "nhwc_packed"], "auto"])
@pytest.mark.parametrize("dtype", [wl.F16, wl.BF16])
def test_config5_stack_with_format_selection(dtype, formats):
    # the same five layers with channel-innermost formats where chosen: conversions by the pools, one explicit
    # conversion (layer 3 -> 4 in the fixed assignment), repacked filters; every layer against the oracle
    torch = torch_mod()
    stack, shapes, gen, x, filts, biases = _stack_on_device(dtype, 20, formats=formats)
    stack.autotune(x, filts, biases)
    say("  formats: %s, filters: %s, pools fused: %s" % (stack.formats, stack.filt_formats, stack.fused))
    if formats == "auto":
        say("  planned total %.1f us" % stack.plan_times["total_us"])
    else:
        assert stack.formats == [f.split("_")[0] for f in formats] and not any(stack.fused)
        assert stack.filt_formats == [{"nchw": "kcrs", "nhwc": "krsc", "nhwc_packed": "packed"}[f] for f in formats]
        for f, d in zip(formats, stack.descs):
            assert B.conv_variant_name(d, -1).startswith("pwin_") == (f == "nhwc_packed")
    assert stack.formats[0] == "nchw"  # three input channels: no channel-innermost kernel
    y = stack.run(x, filts, biases)
    torch.cuda.synchronize()
    _check_stack_against_oracle(stack, shapes, gen, dtype, y)
    # the native schedule (one library call for the chain) and the call-per-operation walk run the same kernels
    want = to_host_stored(y, dtype).copy()
    y.fill_(float("nan"))
    y2 = stack.run_stepwise(x, filts, biases)
    torch.cuda.synchronize()
    assert np.array_equal(to_host_stored(y2, dtype).view(np.uint16), want.view(np.uint16))


def test_config5_format_selection_on_a_side_stream_times_the_glue():
    # the planner times pools and conversions through a captured graph: they must land on the capturing stream also when
    # the caller hands over a stream of its own (an empty graph would make every pool look free)
    torch = torch_mod()
    stack, shapes, gen, x, filts, biases = _stack_on_device(wl.F16, 5, formats="auto")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    stack.autotune(x, filts, biases, stream=side)
    side.synchronize()
    pools = [stack.plan_times["glue_us"][i] for i in (0, 1)]
    assert all(v > 0.5 for g in pools for v in g.values()), pools
    y = stack.run(x, filts, biases, stream=side)
    side.synchronize()
    torch.cuda.synchronize()
    _check_stack_against_oracle(stack, shapes, gen, wl.F16, y)


@pytest.mark.parametrize("dtype", [wl.F16, wl.BF16])
def test_config5_stack_with_the_pools_fused_into_their_convolutions(dtype):
    # fuse_pool fuses every pool that some kernel can run in its epilogue.  The first layer's kernel for this pooling
    # computes tiles of pooled outputs and serves both output layouts; behind layer 2 the pool goes only with
    # channel-innermost layers, whose 768-pixel tiles hold a whole 27x27 image (no [N][C][H][W] kernel does).
    torch = torch_mod()
    planar = ConvStack([w.shape for w in wl.config5_layers(5, dtype)], dtype, pool_after=wl.STACK_POOL_AFTER, fuse_pool=True)
    assert planar.fused == [True, False, False, False, False]
    del planar
    for formats in (None, ["nchw", "nhwc", "nhwc", "nhwc", "nhwc"]):
        stack, shapes, gen, x, filts, biases = _stack_on_device(dtype, 5, formats=formats, fuse_pool=True)
        assert stack.fused == [True, formats is not None, False, False, False]
        stack.autotune(x, filts, biases)
        y = stack.run(x, filts, biases)
        torch.cuda.synchronize()
        _check_stack_against_oracle(stack, shapes, gen, dtype, y)


@pytest.mark.parametrize("formats,fuse_pool", [(None, False), (["nchw", "nhwc", "nhwc", "nhwc", "nhwc"], False),
                                               (["nchw", "nhwc", "nhwc", "nhwc", "nhwc"], True)])
def test_config5_stack_as_hip_graph(formats, fuse_pool):
    """The stack recorded into a HIP graph must reproduce the eagerly enqueued stack bit for bit, on every replay: the
    graph is replayed several times with eager runs, buffer poisoning and synchronisations in between."""
    torch = torch_mod()
    dtype = wl.F16
    layers = wl.config5_layers(5, dtype)
    shapes = [w.shape for w in layers]
    stack = ConvStack(shapes, dtype, pool_after=wl.STACK_POOL_AFTER, formats=formats, fuse_pool=fuse_pool)
    assert any(stack.fused) == fuse_pool
    gen = [w.generate() for w in layers]
    x = to_device(gen[0]["in"], dtype)
    filts = [to_device(g["filt"], dtype) for g in gen]
    biases = [to_device(g["bias"], wl.F32) for g in gen]
    stack.autotune(x, filts, biases)
    last = len(shapes) - 1

    def snapshot():
        torch.cuda.synchronize()
        return [to_host_stored(stack.layer_output(i), dtype).copy() for i in range(len(shapes))]

    def poison():
        for i in range(len(shapes)):
            for t in (stack.conv_out[i], stack.pool_out[i], stack.convert_out[i]):
                if t is not None:
                    t.fill_(float("nan"))

    stack.run(x, filts, biases)
    eager = snapshot()
    assert np.all(np.isfinite(wl.storage_to_f64(eager[last], dtype)))
    graph = stack.capture(x, filts, biases)
    for rep in range(4):
        poison()
        if rep % 2:
            stack.run(x, filts, biases)     # eager work of the same program between replays
            torch.cuda.synchronize()
            poison()
        graph.replay()
        got = snapshot()
        for i in range(len(shapes)):
            assert np.array_equal(got[i], eager[i]), "replay %d, layer %d differs from the eager run" % (rep, i + 1)
    say("  %s: 4 graph replays identical to the eager run" % (stack.formats,))
