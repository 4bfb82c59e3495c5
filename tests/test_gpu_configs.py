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
