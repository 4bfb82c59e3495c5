"""Pins of the CPU oracle against things other than itself (CPU only).

Each test fixes a part of the definition that a plausible slip would break:
a dropped term, a flipped filter, a wrong pad or stride, a transposed index,
bias after the activation, ceil instead of floor in the output size.
"""
import itertools
import math

import numpy as np
import pytest

import oracle
from paper_1611_06945_amd.workloads import ConvShape


def brute_force(inp, filt, bias, stride, pad, relu):
    """Independent literal evaluation with Python loops and Python integers/floats."""
    N, C, H, W = inp.shape
    K, _, R, S = filt.shape
    OH = (H + 2 * pad - R) // stride + 1
    OW = (W + 2 * pad - S) // stride + 1
    out = np.zeros((N, K, OH, OW), dtype=np.float64)
    for n, k, oy, ox in itertools.product(range(N), range(K), range(OH), range(OW)):
        acc = 0.0
        for c, r, s in itertools.product(range(C), range(R), range(S)):
            iy, ix = oy * stride - pad + r, ox * stride - pad + s
            if 0 <= iy < H and 0 <= ix < W:
                acc += float(inp[n, c, iy, ix]) * float(filt[k, c, r, s])
        if bias is not None:
            acc += float(bias[k])
        if relu:
            acc = max(acc, 0.0)
        out[n, k, oy, ox] = acc
    return out


def window_view_conv(inp, filt, stride, pad):
    """Second independent route: explicit zero-padded copy + strided window view + einsum."""
    N, C, H, W = inp.shape
    K, _, R, S = filt.shape
    xp = np.zeros((N, C, H + 2 * pad, W + 2 * pad), dtype=np.float64)
    xp[:, :, pad:pad + H, pad:pad + W] = inp
    win = np.lib.stride_tricks.sliding_window_view(xp, (R, S), axis=(2, 3))[:, :, ::stride, ::stride]
    return np.einsum("ncyxrs,kcrs->nkyx", win, filt.astype(np.float64))


@pytest.mark.parametrize("stride", [1, 2, 3])
@pytest.mark.parametrize("pad", [0, 1, 2])
@pytest.mark.parametrize("relu", [False, True])
def test_brute_force_small_integers_exact(stride, pad, relu):
    rng = np.random.default_rng(100 * stride + 10 * pad + relu)
    inp = rng.integers(-3, 4, size=(2, 3, 5, 6)).astype(np.float64)
    filt = rng.integers(-2, 3, size=(4, 3, 3, 2)).astype(np.float64)  # R != S on purpose
    bias = rng.integers(-4, 5, size=(4,)).astype(np.float64)
    got = oracle.conv_fwd(inp, filt, bias, stride=stride, pad=pad, relu=relu)
    ref = brute_force(inp, filt, bias, stride, pad, relu)
    assert got.shape == ref.shape
    assert np.array_equal(got, ref)


@pytest.mark.parametrize("geom", [(7, 9, 3, 3, 1, 1), (8, 8, 5, 5, 2, 2), (9, 7, 2, 4, 3, 0), (6, 6, 6, 6, 1, 0),
                                  (5, 5, 1, 1, 2, 0), (4, 5, 3, 3, 1, 3)])
def test_window_view_route_random_floats(geom):
    H, W, R, S, stride, pad = geom
    rng = np.random.default_rng(7)
    inp = rng.normal(size=(2, 3, H, W))
    filt = rng.normal(size=(5, 3, R, S))
    got = oracle.conv_fwd(inp, filt, None, stride=stride, pad=pad)
    ref = window_view_conv(inp, filt, stride, pad)
    assert got.shape == ref.shape
    assert np.max(np.abs(got - ref)) < 1e-12


def test_pad_not_smaller_than_window_is_legal():
    # pad >= R: border outputs see padding only and equal act(bias) (geometry (4,5,3,3,1,3) above is one such).
    inp = np.ones((1, 1, 2, 2))
    filt = np.ones((1, 1, 2, 2))
    out = oracle.conv_fwd(inp, filt, np.array([-1.5]), stride=1, pad=2, relu=False)
    assert out.shape == (1, 1, 5, 5)
    assert out[0, 0, 0, 0] == -1.5 and out[0, 0, 4, 4] == -1.5
    assert out[0, 0, 2, 2] == 4 - 1.5


@pytest.mark.parametrize("R", [1, 3, 5])
def test_identity_filter_returns_input(R):
    rng = np.random.default_rng(R)
    C = 4
    inp = rng.normal(size=(2, C, 6, 7))
    filt = np.zeros((C, C, R, R))
    for c in range(C):
        filt[c, c, R // 2, R // 2] = 1.0
    out = oracle.conv_fwd(inp, filt, None, stride=1, pad=R // 2)
    assert np.array_equal(out, inp)
    out = oracle.conv_fwd(inp, filt, None, stride=1, pad=R // 2, relu=True)
    assert np.array_equal(out, np.maximum(inp, 0.0))


@pytest.mark.parametrize("r0,s0", [(0, 0), (0, 2), (2, 1), (1, 0)])
def test_shifted_delta_pins_orientation_and_zero_fill(r0, s0):
    # A delta at (r0, s0) must read in[y - pad + r0, x - pad + s0]: no flip of the filter.
    rng = np.random.default_rng(11)
    H, W, pad = 5, 6, 1
    inp = rng.normal(size=(1, 2, H, W))
    filt = np.zeros((2, 2, 3, 3))
    filt[0, 1, r0, s0] = 1.0  # output channel 0 reads input channel 1
    filt[1, 0, r0, s0] = 1.0  # and the other way round: pins the (k, c) order as well
    out = oracle.conv_fwd(inp, filt, None, stride=1, pad=pad)
    exp = np.zeros_like(out)
    for y in range(H):
        for x in range(W):
            iy, ix = y - pad + r0, x - pad + s0
            if 0 <= iy < H and 0 <= ix < W:
                exp[0, 0, y, x] = inp[0, 1, iy, ix]
                exp[0, 1, y, x] = inp[0, 0, iy, ix]
    assert np.array_equal(out, exp)


def test_pointwise_is_a_matrix_product():
    rng = np.random.default_rng(5)
    N, C, H, W, K = 3, 7, 4, 5, 6
    inp = rng.normal(size=(N, C, H, W))
    wgt = rng.normal(size=(K, C))
    out = oracle.conv_fwd(inp, wgt.reshape(K, C, 1, 1), None)
    for n in range(N):
        ref = wgt @ inp[n].reshape(C, H * W)
        assert np.max(np.abs(out[n].reshape(K, H * W) - ref)) < 1e-13
    # stride-2 pointwise == subsample, then matrix product
    out2 = oracle.conv_fwd(inp, wgt.reshape(K, C, 1, 1), None, stride=2)
    sub = inp[:, :, ::2, ::2]
    assert out2.shape == (N, K) + sub.shape[2:]
    for n in range(N):
        ref = wgt @ sub[n].reshape(C, -1)
        assert np.max(np.abs(out2[n].reshape(K, -1) - ref)) < 1e-13


def test_full_size_filter_is_a_dot_product():
    # The fully-connected-as-convolution case of the paper (Section 4; Appendix A row 6x6x256 -> 1x1x4096), scaled down.
    rng = np.random.default_rng(6)
    N, C, H, W, K = 2, 5, 6, 6, 9
    inp = rng.normal(size=(N, C, H, W))
    filt = rng.normal(size=(K, C, H, W))
    bias = rng.normal(size=(K,))
    out = oracle.conv_fwd(inp, filt, bias)
    assert out.shape == (N, K, 1, 1)
    ref = inp.reshape(N, -1) @ filt.reshape(K, -1).T + bias
    assert np.max(np.abs(out.reshape(N, K) - ref)) < 1e-12


def test_linearity_in_input_and_in_filter():
    rng = np.random.default_rng(8)
    x, y = rng.normal(size=(2, 2, 3, 6, 5))
    w, v = rng.normal(size=(2, 4, 3, 3, 3))
    a, b = 1.75, -0.625
    f = lambda i, g: oracle.conv_fwd(i, g, None, stride=2, pad=1)
    assert np.max(np.abs(f(a * x + b * y, w) - (a * f(x, w) + b * f(y, w)))) < 1e-12
    assert np.max(np.abs(f(x, a * w + b * v) - (a * f(x, w) + b * f(x, v)))) < 1e-12


@pytest.mark.parametrize("H,W,R,S,stride,pad", [(6, 7, 3, 3, 1, 1), (9, 8, 5, 3, 2, 2), (7, 7, 3, 3, 3, 0), (5, 4, 4, 2, 1, 3)])
def test_all_ones_closed_form(H, W, R, S, stride, pad):
    C, K = 3, 2
    out = oracle.conv_fwd(np.ones((1, C, H, W)), np.ones((K, C, R, S)), None, stride=stride, pad=pad)
    OH, OW = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    assert out.shape == (1, K, OH, OW)
    for oy in range(OH):
        ny = sum(1 for r in range(R) if 0 <= oy * stride - pad + r < H)
        for ox in range(OW):
            nx = sum(1 for s in range(S) if 0 <= ox * stride - pad + s < W)
            assert out[0, 0, oy, ox] == C * ny * nx
            assert out[0, 1, oy, ox] == C * ny * nx


def test_zero_input_gives_activation_of_bias_and_relu_follows_bias():
    K = 5
    bias = np.array([-2.0, -0.5, 0.0, 0.25, 3.0])
    filt = np.random.default_rng(2).normal(size=(K, 2, 3, 3))
    out = oracle.conv_fwd(np.zeros((2, 2, 4, 4)), filt, bias, pad=1, relu=True)
    for k in range(K):
        assert np.all(out[:, k] == max(bias[k], 0.0))
    out = oracle.conv_fwd(np.zeros((2, 2, 4, 4)), filt, bias, pad=1, relu=False)
    for k in range(K):
        assert np.all(out[:, k] == bias[k])
    # bias is added before the activation: conv = -1 everywhere, bias = +3 -> 2, not 3
    o = oracle.conv_fwd(np.ones((1, 1, 3, 3)), -np.ones((1, 1, 1, 1)), np.array([3.0]), relu=True)
    assert np.all(o == 2.0)
    # negated filter on a positive input is clipped to zero
    pos = np.abs(np.random.default_rng(3).normal(size=(1, 2, 5, 5))) + 0.1
    o = oracle.conv_fwd(pos, -np.abs(filt) - 0.1, None, pad=1, relu=True)
    assert np.all(o == 0.0)


def test_output_sizes_and_flops_of_appendix_a(appendix_a):
    assert len(appendix_a) == 43
    for row in appendix_a:
        oh, ow = oracle.conv_out_shape(row["in_y"], row["in_x"], row["ksz"], row["ksz"], row["stride"], row["pad"])
        assert (oh, ow) == (row["out_y"], row["out_x"]), row
        assert row["oc"] == row["out_c"]
        sh = ConvShape(row["b"], row["in_c"], row["in_y"], row["in_x"], row["oc"], row["ksz"], row["ksz"],
                       row["stride"], row["pad"])
        assert (sh.OH, sh.OW) == (oh, ow)
        # FLOP convention 2*B*OH*OW*OC*IC*KSZ^2, printed with six significant digits
        assert "%.6g" % sh.flops == "%.6g" % row["flops"], (row, sh.flops)
        assert abs(sh.flops - row["flops"]) <= 5e-6 * row["flops"]


def test_floor_rounding_cases_named_in_the_table():
    assert oracle.conv_out_shape(227, 227, 11, 11, 4, 0) == (55, 55)
    assert oracle.conv_out_shape(224, 224, 11, 11, 4, 0) == (54, 54)  # 54.25 -> 54
    assert oracle.conv_out_shape(224, 224, 7, 7, 2, 3) == (112, 112)  # 112.5 -> 112
    assert oracle.conv_out_shape(27, 27, 5, 5, 1, 2) == (27, 27)
    assert oracle.conv_out_shape(13, 13, 3, 3, 1, 1) == (13, 13)
    assert oracle.conv_out_shape(6, 6, 6, 6, 1, 0) == (1, 1)
    with pytest.raises(ValueError):
        oracle.conv_out_shape(4, 4, 5, 5, 1, 0)


def test_points_agree_with_full_output():
    rng = np.random.default_rng(21)
    inp = rng.normal(size=(2, 3, 9, 8))
    filt = rng.normal(size=(4, 3, 3, 2))
    bias = rng.normal(size=(4,))
    full = oracle.conv_fwd(inp, filt, bias, stride=2, pad=1, relu=True)
    idx = rng.integers(0, full.size, size=50)
    vals = oracle.conv_fwd_points(inp, filt, bias, idx, stride=2, pad=1, relu=True)
    assert np.array_equal(vals, full.reshape(-1)[idx])
    with pytest.raises(ValueError):
        oracle.conv_fwd_points(inp, filt, bias, [full.size], stride=2, pad=1)


def test_maxpool_against_loops_and_known_values():
    rng = np.random.default_rng(4)
    inp = rng.normal(size=(2, 3, 9, 11))
    out = oracle.maxpool_fwd(inp, win=3, stride=2)
    assert out.shape == (2, 3, 4, 5)
    for n, c, oy, ox in itertools.product(range(2), range(3), range(4), range(5)):
        assert out[n, c, oy, ox] == max(inp[n, c, 2 * oy + r, 2 * ox + s] for r in range(3) for s in range(3))
    ramp = np.arange(25, dtype=np.float64).reshape(1, 1, 5, 5)
    assert np.array_equal(oracle.maxpool_fwd(ramp, win=3, stride=2).reshape(2, 2), [[12, 14], [22, 24]])
    # the two pools of the five-layer stack: 55 -> 27 and 27 -> 13
    assert oracle.maxpool_fwd(np.zeros((1, 1, 55, 55))).shape[2:] == (27, 27)
    assert oracle.maxpool_fwd(np.zeros((1, 1, 27, 27))).shape[2:] == (13, 13)
    # all-negative input: the maximum is not clipped at zero
    assert np.all(oracle.maxpool_fwd(-np.ones((1, 1, 3, 3))) == -1.0)


def test_error_metric():
    ref = np.array([1.0, -4.0, 2.0])
    assert oracle.max_normalised_error(ref, ref) == 0.0
    assert math.isclose(oracle.max_normalised_error(ref + np.array([0.0, 0.0, 0.02]), ref), 0.005)
