"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element.

Tolerances (max normalised error, oracle.max_normalised_error): 1e-5 for fp32, 5e-3 for fp16/bf16 storage.
Small-integer cases must match bit for bit whatever the tile shape, split or accumulation order.
"""
import sys

import numpy as np
import pytest

import oracle
from paper_1611_06945_amd import binding as B
from paper_1611_06945_amd import workloads as wl
from paper_1611_06945_amd.workloads import ConvShape

from gpu_util import TOL, DeviceCase, empty_out, to_device, to_host_f64, to_host_stored, torch_mod

pytestmark = pytest.mark.gpu

DTYPES = [wl.F32, wl.F16, wl.BF16]


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def random_case(shape, dtype, seed, relu=True, use_bias=True):
    data = {
        "in": wl.to_storage(wl.draw(("uniform", -1.0, 1.0), shape.in_shape(), seed), dtype),
        "filt": wl.to_storage(wl.draw(("normal", wl.he_sigma(shape)), shape.filt_shape(), seed + 1), dtype),
        "bias": wl.draw(("uniform", -0.1, 0.1), (shape.K,), seed + 2),
    }
    return DeviceCase(shape, dtype, data, relu=relu, use_bias=use_bias)


def int_case(shape, dtype, seed, relu=True, use_bias=True):
    return DeviceCase(shape, dtype, wl.small_int_case(shape, dtype, seed), relu=relu, use_bias=use_bias)


def assert_bit_exact(case, out, what):
    exp = wl.storage_to_f64(wl.to_storage(case.ref().astype(np.float32), case.dtype), case.dtype)
    got = to_host_f64(out, case.dtype)
    bad = np.argwhere(got != exp)
    assert bad.size == 0, "%s: %d mismatches, first at %s got %r want %r" % (
        what, len(bad), tuple(bad[0]), got[tuple(bad[0])], exp[tuple(bad[0])])


# Shapes small enough for the oracle to finish at once, large enough to span several tiles in each GEMM
# dimension with ragged tails (K, P and C*R*S are not tile multiples).
SMALL_SHAPES = [
    ConvShape(2, 8, 9, 11, 40, 3, 3, 1, 1),     # C*R*S = 72: 16-byte filter loads valid for every type
    ConvShape(3, 3, 19, 17, 20, 5, 4, 2, 2),    # C*R*S = 60: vector loads valid for fp32 only; R != S, stride 2
    ConvShape(1, 3, 32, 32, 16, 3, 3, 1, 1),    # benchmark configuration 1: C*R*S = 27, element-wise loads only
    ConvShape(3, 24, 6, 10, 50, 1, 1, 1, 0),    # pointwise, H*W % 4 == 0
    ConvShape(2, 20, 12, 12, 200, 3, 3, 1, 1),  # K spans two 128-row tiles; 180-long reduction allows splits
    ConvShape(2, 5, 23, 23, 96, 7, 7, 4, 0),    # first-layer like: few channels, big window, stride 4, K = 96
    ConvShape(3, 64, 13, 13, 40, 3, 3, 1, 1),   # window-reuse kernel: 169 pixels per image, 4 channel chunks, ragged K
    ConvShape(2, 32, 15, 15, 33, 3, 3, 1, 0),   # window-reuse kernel without padding (13x13 outputs)
    ConvShape(2, 48, 12, 16, 16, 3, 3, 1, 1),   # window-reuse kernel, non-square image (192 pixels -> 13 blocks)
    ConvShape(1, 32, 10, 11, 20, 3, 3, 1, 2),   # window-reuse kernel, pad 2 (12x13 outputs)
    ConvShape(2, 32, 27, 27, 40, 5, 5, 1, 2),   # 16-bit window kernel, 5x5: four bands of rows per image, last one partial
    ConvShape(1, 64, 20, 20, 33, 3, 3, 1, 1),   # 16-bit window kernel, 3x3: bands of 9, 9 and 2 rows
    ConvShape(5, 16, 6, 6, 70, 6, 6, 1, 0),     # fully connected (window = image), 5 images, K ragged against the row blocks
    ConvShape(3, 1032, 1, 1, 33, 1, 1, 1, 0),   # fully connected 1x1 on 1x1: 258 / 129 vectors against 256 threads
    ConvShape(8, 24, 2, 2, 10, 2, 2, 1, 0),     # fully connected, 8 images
    ConvShape(4, 16, 7, 9, 24, 5, 5, 1, 2),     # fp32 window kernel with channel-waves, 5x5: chunks of 8 channels, pixel tiles straddle images
    ConvShape(3, 72, 6, 10, 50, 1, 1, 1, 0),    # pointwise with the channels split over the waves of a workgroup: 9 groups of 8 channels over 4 or 8 waves, ragged K and pixel tiles
    ConvShape(2, 136, 5, 7, 100, 1, 1, 1, 0),   # the same over 16 waves (17 groups), tiles straddle images, odd row length
    ConvShape(3, 144, 6, 10, 50, 1, 1, 1, 0),   # the same in 16-bit storage: 9 groups of 16 channels over 4 or 8 waves
    ConvShape(2, 272, 5, 7, 100, 1, 1, 1, 0),   # 17 groups of 16 channels over 16 waves, odd row length (2-byte rows at odd offsets)
]


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("si", range(len(SMALL_SHAPES)))
def test_every_variant_small_shapes(si, dtype):
    shape = SMALL_SHAPES[si]
    icase = int_case(shape, dtype, 500 + si)
    rcase = random_case(shape, dtype, 600 + si)
    names = icase.variant_names()
    assert names, "no variant for %s" % (shape,)
    for vi, name in enumerate(names):
        say("  variant %s on %s dtype %d" % (name, shape, dtype))
        assert_bit_exact(icase, icase.run(variant=vi), name)
        err = rcase.error(rcase.run(variant=vi))
        assert err <= TOL[dtype], "%s: error %.3g" % (name, err)


EDGE_SHAPES = [
    (ConvShape(1, 1, 1, 1, 1, 1, 1, 1, 0), "single element"),
    (ConvShape(2, 3, 2, 2, 5, 2, 2, 1, 2), "pad >= window: border outputs are act(bias)"),
    (ConvShape(2, 4, 7, 9, 6, 7, 9, 1, 0), "full-size filter: one output per image and channel"),
    (ConvShape(1, 6, 10, 7, 9, 1, 1, 2, 0), "pointwise with stride 2 (not the pointwise fast path)"),
    (ConvShape(1, 6, 5, 7, 9, 1, 1, 1, 0), "pointwise with H*W % 4 != 0"),
    (ConvShape(2, 2, 11, 13, 3, 3, 5, 3, 1), "stride 3, R != S"),
    (ConvShape(1, 1, 40, 40, 1, 3, 3, 1, 1), "one channel in, one out"),
    (ConvShape(1, 64, 1, 300, 33, 1, 3, 1, 1), "height 1"),
    (ConvShape(5, 7, 3, 3, 130, 3, 3, 1, 1), "K just over one 128 tile"),
]


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("ei", range(len(EDGE_SHAPES)))
def test_edge_shapes_default_selection(ei, dtype):
    shape, why = EDGE_SHAPES[ei]
    for relu, use_bias in [(True, True), (False, True), (True, False), (False, False)]:
        case = int_case(shape, dtype, 700 + ei, relu=relu, use_bias=use_bias)
        say("  %s: %s relu=%s bias=%s -> %s" % (why, shape, relu, use_bias, B.conv_variant_name(case.desc, -1)))
        assert_bit_exact(case, case.run(with_ws=True), why)
        assert_bit_exact(case, case.run(with_ws=False), why + " (no workspace)")


@pytest.mark.parametrize("dtype", DTYPES)
def test_identity_and_shifted_delta_filters(dtype):
    # identity filter returns the stored input bit for bit; a delta off centre pins the window orientation on the GPU
    shape = ConvShape(2, 16, 13, 13, 16, 3, 3, 1, 1)
    x32 = wl.draw(("uniform", -2.0, 2.0), shape.in_shape(), 42)
    x32[np.abs(x32) < 0.05] = 0.5  # keep clear of zeros and 16-bit subnormals: signed zeros would blur "bit for bit"
    x = wl.to_storage(x32, dtype)
    for (r0, s0) in [(1, 1), (0, 2), (2, 0)]:
        f = np.zeros(shape.filt_shape(), dtype=np.float32)
        for c in range(16):
            f[c, c, r0, s0] = 1.0
        case = DeviceCase(shape, dtype, {"in": x, "filt": wl.to_storage(f, dtype), "bias": np.zeros(16, np.float32)},
                          relu=False, use_bias=False)
        for vi, name in enumerate(case.variant_names()):
            got = to_host_f64(case.run(variant=vi), dtype)
            if name.startswith("wino_"):
                # the Winograd variants add and subtract neighbouring inputs before multiplying: on arbitrary floats a
                # delta filter comes back within round-off, not bit for bit (a wrong orientation would be a gross error)
                assert oracle.max_normalised_error(got, case.ref()) <= TOL[dtype], (name, r0, s0)
            else:
                assert np.array_equal(got, case.ref()), (name, r0, s0)
    f = np.zeros(shape.filt_shape(), dtype=np.float32)
    for c in range(16):
        f[c, c, 1, 1] = 1.0
    case = DeviceCase(shape, dtype, {"in": x, "filt": wl.to_storage(f, dtype), "bias": np.zeros(16, np.float32)},
                      relu=False, use_bias=False)
    assert np.array_equal(to_host_stored(case.run(), dtype), x)


def test_zero_input_gives_relu_of_bias():
    shape = ConvShape(2, 8, 6, 6, 12, 3, 3, 1, 1)
    for dtype in DTYPES:
        data = wl.small_int_case(shape, dtype, 9)
        data["in"] = wl.to_storage(np.zeros(shape.in_shape(), np.float32), dtype)
        case = DeviceCase(shape, dtype, data)
        got = to_host_f64(case.run(), dtype)
        for k in range(shape.K):
            assert np.all(got[:, k] == max(float(data["bias"][k]), 0.0))


@pytest.mark.parametrize("dtype", DTYPES)
def test_split_variants_are_deterministic(dtype):
    shape = ConvShape(2, 20, 12, 12, 200, 3, 3, 1, 1)
    case = random_case(shape, dtype, 77)
    split = [i for i, n in enumerate(case.variant_names()) if "_sk" in n]
    assert split
    for vi in split[:6]:
        a = to_host_stored(case.run(variant=vi), dtype)
        b = to_host_stored(case.run(variant=vi), dtype)
        assert np.array_equal(a, b)


def test_forced_split_variant_without_workspace_is_an_error():
    shape = ConvShape(2, 20, 12, 12, 200, 3, 3, 1, 1)
    case = random_case(shape, wl.F32, 78)
    vi = next(i for i, n in enumerate(case.variant_names()) if "_sk" in n)
    B.conv_force_variant(case.desc, vi)
    try:
        out = empty_out(shape.out_shape(), wl.F32)
        with pytest.raises(B.ConvError) as e:
            B.conv_fwd(case.desc, case.d_in, case.d_filt, case.d_bias, out)
        assert e.value.status == B.CONV_EWORKSPACE
    finally:
        B.conv_force_variant(case.desc, -1)


@pytest.mark.parametrize("dtype", DTYPES)
def test_maxpool_bit_exact(dtype):
    torch = torch_mod()
    for (N, C, H, W, win, stride) in [(2, 5, 55, 55, 3, 2), (3, 7, 27, 27, 3, 2), (1, 3, 9, 11, 2, 1), (2, 2, 8, 8, 2, 2)]:
        x = wl.to_storage(wl.draw(("normal", 1.0), (N, C, H, W), 5), dtype)
        ref = oracle.maxpool_fwd(wl.storage_to_f64(x, dtype), win=win, stride=stride)
        out = empty_out(ref.shape, dtype)
        B.maxpool_fwd(N, C, H, W, win, stride, dtype, to_device(x, dtype), out)
        torch.cuda.synchronize()
        assert np.array_equal(to_host_f64(out, dtype), ref)


def test_autotune_records_times_and_selects_the_fastest():
    B.conv_cache_clear()
    case = random_case(ConvShape(2, 20, 12, 12, 200, 3, 3, 1, 1), wl.F32, 80)
    out = empty_out(case.shape.out_shape(), wl.F32)
    ws = case.workspace()
    B.conv_autotune(case.desc, case.d_in, case.d_filt, case.d_bias, out, ws, ws.numel())
    n = B.conv_variant_count(case.desc)
    times = [B.conv_variant_time_us(case.desc, i) for i in range(n)]
    assert all(t > 0 for t in times), times
    names = case.variant_names()
    assert B.conv_variant_name(case.desc, -1) == names[int(np.argmin(times))]
    nows = [i for i in range(n) if B.conv_variant_workspace(case.desc, i) == 0]
    assert B.conv_variant_name(case.desc, -2) == names[min(nows, key=lambda i: times[i])]
    # what the autotuner left selected still computes the right thing
    assert case.error(case.run()) <= TOL[wl.F32]
    assert case.error(case.run(with_ws=False)) <= TOL[wl.F32]
    B.conv_cache_clear()


@pytest.mark.parametrize("dtype", DTYPES)
def test_compare_outputs_is_the_parity_metric(dtype):
    torch = torch_mod()
    rng = np.random.default_rng(77)
    ref = wl.to_storage(rng.normal(0.0, 1.0, 70001).astype(np.float32), dtype)
    got = ref.copy()
    d_ref, d_got = to_device(ref, dtype), to_device(got, dtype)
    assert B.conv_compare_outputs(dtype, d_got, d_ref, ref.size) == 0.0
    # one element moved by a known amount, near the end of the tensor (past every whole block of threads)
    r64 = wl.storage_to_f64(ref, dtype)
    g64 = r64.copy()
    g64[69990] += 0.25
    got = wl.to_storage(g64.astype(np.float32), dtype)
    want = oracle.max_normalised_error(wl.storage_to_f64(got, dtype), r64)
    err = B.conv_compare_outputs(dtype, to_device(got, dtype), d_ref, ref.size)
    assert want > 0.01 and abs(err - want) <= 1e-6 * want, (err, want)
    # a NaN or an infinity in the tested tensor is an infinite error, wherever it sits
    for bad in (np.nan, np.inf):
        g64 = r64.copy()
        g64[12345] = bad
        err = B.conv_compare_outputs(dtype, to_device(wl.to_storage(g64.astype(np.float32), dtype), dtype), d_ref, ref.size)
        assert err == float("inf")
    torch.cuda.synchronize()


def test_autotune_rejects_a_candidate_whose_output_is_wrong(monkeypatch):
    # the candidate named by the test hook gets its output overwritten from the host before the cross-check: it must be
    # neither timed nor selected, even though it would otherwise be eligible; everything else is unaffected
    B.conv_cache_clear()
    case = random_case(ConvShape(2, 20, 12, 12, 200, 3, 3, 1, 1), wl.F32, 82)
    out = empty_out(case.shape.out_shape(), wl.F32)
    ws = case.workspace()
    B.conv_autotune(case.desc, case.d_in, case.d_filt, case.d_bias, out, ws, ws.numel())
    names = case.variant_names()
    winner = B.conv_variant_name(case.desc, -1)
    assert all(B.conv_variant_time_us(case.desc, i) > 0 for i in range(len(names)))  # nothing rejected on a clean run
    B.conv_cache_clear()
    monkeypatch.setenv("CONVFWD_AUTOTUNE_CORRUPT", winner)
    B.conv_autotune(case.desc, case.d_in, case.d_filt, case.d_bias, out, ws, ws.numel())
    monkeypatch.delenv("CONVFWD_AUTOTUNE_CORRUPT")
    times = [B.conv_variant_time_us(case.desc, i) for i in range(len(names))]
    wi = names.index(winner)
    if wi == 0:
        pytest.skip("the fastest variant is the cross-check's own reference")
    assert times[wi] == -2.0, times[wi]
    assert all(t > 0 for i, t in enumerate(times) if i != wi)
    assert B.conv_variant_name(case.desc, -1) != winner
    assert case.error(case.run()) <= TOL[wl.F32]
    B.conv_cache_clear()


def test_device_side_timing_entry_point():
    case = random_case(ConvShape(2, 20, 12, 12, 200, 3, 3, 1, 1), wl.F32, 81)
    out = empty_out(case.shape.out_shape(), wl.F32)
    ws = case.workspace()
    us = B.conv_time_us(case.desc, case.d_in, case.d_filt, case.d_bias, out, ws, ws.numel(), launches=20)
    assert 0.5 < us < 1e4, us
    torch_mod().cuda.synchronize()
    assert case.error(out) <= TOL[wl.F32]  # the timed launches compute the real thing
