"""GPU parity of the 3x3 stride-2 max-pool fused into the convolution's epilogue (CONV_FLAG_MAXPOOL_3X3S2): against the
CPU oracle's convolution followed by its max-pool, and bit for bit against the library's own two-call sequence."""
import numpy as np
import pytest

import oracle
from paper_1611_06945_amd import binding as B
from paper_1611_06945_amd import workloads as wl
from paper_1611_06945_amd.workloads import ConvShape

from gpu_util import TOL, empty_out, to_device, to_host_f64, to_host_stored, torch_mod
from test_gpu_parity import say

pytestmark = pytest.mark.gpu

DT16 = [wl.F16, wl.BF16]


def nhwc(a):
    return np.ascontiguousarray(np.transpose(a, (0, 2, 3, 1)))


def nchw(a):
    return np.ascontiguousarray(np.transpose(a, (0, 3, 1, 2)))


POOL_SHAPES = [
    ConvShape(3, 64, 13, 13, 40, 3, 3, 1, 1),    # 13x13 -> 6x6, K ragged against the 32-row blocks
    ConvShape(2, 32, 14, 12, 64, 3, 3, 1, 1),    # 14x12 -> 6x5: even extents leave the last row and column unused
    ConvShape(2, 32, 13, 13, 33, 3, 3, 1, 0),    # no padding: 11x11 -> 5x5
    ConvShape(2, 32, 5, 42, 8, 3, 3, 1, 0),      # 3x40 -> 1x19: a single row of windows (planar kernels only)
    ConvShape(2, 32, 13, 13, 40, 5, 5, 1, 2),    # 5x5 window
    ConvShape(1, 16, 27, 27, 48, 5, 5, 1, 2),    # 27x27 -> 13x13: only the 768-pixel tiles hold the whole image
]


def data_for(shape, dtype, seed, ints):
    if ints:
        return wl.small_int_case(shape, dtype, seed)
    return {
        "in": wl.to_storage(wl.draw(("uniform", -1.0, 1.0), shape.in_shape(), seed), dtype),
        "filt": wl.to_storage(wl.draw(("normal", wl.he_sigma(shape)), shape.filt_shape(), seed + 1), dtype),
        "bias": wl.draw(("uniform", -0.1, 0.1), (shape.K,), seed + 2),
    }


def run(desc, d_in, d_filt, d_bias, oshape, dtype, variant):
    torch = torch_mod()
    out = empty_out(oshape, dtype)
    ws = torch.empty(max(256, B.conv_workspace_bytes(desc)), dtype=torch.uint8, device="cuda")
    B.conv_force_variant(desc, variant)
    try:
        B.conv_fwd_ws(desc, d_in, d_filt, d_bias, out, ws, ws.numel())
        torch.cuda.synchronize()
    finally:
        B.conv_force_variant(desc, -1)
    return out


def _served(si, layout):
    """Combinations some kernel serves: channel-innermost outputs need K % 8 == 0; no planar window kernel holds an image
    of more than 192 pixels in one tile; the channel-innermost kernels have no staging slots for the 42-wide rows."""
    shape = POOL_SHAPES[si]
    if layout == "nhwc_to_nhwc" and shape.K % 8:
        return False
    if layout == "planar" and shape.OH * shape.OW > 192:
        return False
    if layout != "planar" and shape.H == 5:
        return False
    return True


POOL_CASES = [(si, layout) for si in range(len(POOL_SHAPES)) for layout in ("planar", "nhwc_to_nhwc", "nhwc_to_planar")
              if _served(si, layout)]


@pytest.mark.parametrize("dtype", DT16)
@pytest.mark.parametrize("si,layout", POOL_CASES)
def test_fused_maxpool_every_variant(si, layout, dtype):
    torch = torch_mod()
    shape = POOL_SHAPES[si]
    in_nhwc, out_nhwc = layout != "planar", layout == "nhwc_to_nhwc"
    PH, PW = (shape.OH - 3) // 2 + 1, (shape.OW - 3) // 2 + 1
    for ints, relu, use_bias in [(True, True, True), (True, False, False), (False, True, True)]:
        data = data_for(shape, dtype, 3000 + 10 * si, ints)
        conv = oracle.conv_fwd(wl.storage_to_f64(data["in"], dtype), wl.storage_to_f64(data["filt"], dtype),
                               data["bias"].astype(np.float64) if use_bias else None,
                               stride=shape.stride, pad=shape.pad, relu=relu)
        want = oracle.maxpool_fwd(conv, win=3, stride=2)
        assert want.shape == (shape.N, shape.K, PH, PW)
        d_in = to_device(nhwc(data["in"]) if in_nhwc else data["in"], dtype)
        d_filt = to_device(nhwc(data["filt"]) if in_nhwc else data["filt"], dtype)
        d_bias = to_device(data["bias"], wl.F32) if use_bias else None
        kw = dict(relu=relu, in_nhwc=in_nhwc, out_nhwc=out_nhwc, filt_krsc=in_nhwc)
        fused = B.desc_of(shape, dtype, maxpool=True, **kw)
        assert B.conv_out_shape(fused) == (PH, PW)
        names = [B.conv_variant_name(fused, i) for i in range(B.conv_variant_count(fused))]
        assert names, "no variant pools %s (%s)" % (shape, layout)
        plain = B.desc_of(shape, dtype, **kw)
        plain_names = [B.conv_variant_name(plain, i) for i in range(B.conv_variant_count(plain))]
        oshape = (shape.N, PH, PW, shape.K) if out_nhwc else (shape.N, shape.K, PH, PW)
        for vi, name in enumerate(names):
            say("  %s on %s dtype %d %s ints=%s relu=%s bias=%s" % (name, shape, dtype, layout, ints, relu, use_bias))
            out = run(fused, d_in, d_filt, d_bias, oshape, dtype, vi)
            got_bits = to_host_stored(out, dtype)
            # the library's own two-call sequence with the same kernel (same summation order): equal bit for bit
            full = run(plain, d_in, d_filt, d_bias,
                       (shape.N, shape.OH, shape.OW, shape.K) if out_nhwc else shape.out_shape(), dtype, plain_names.index(name))
            seq = empty_out(oshape, dtype)
            B.maxpool_fwd_layout(shape.N, shape.K, shape.OH, shape.OW, 3, 2, dtype, out_nhwc, out_nhwc, full, seq)
            torch.cuda.synchronize()
            seq_bits = to_host_stored(seq, dtype)
            assert np.array_equal(got_bits.view(np.uint16), seq_bits.view(np.uint16)), "%s: differs from conv + maxpool" % name
            got = to_host_f64(out, dtype)
            got = nchw(got) if out_nhwc else got
            assert np.all(np.isfinite(got)), "%s: unwritten or overflowed elements" % name
            if ints:
                exp = wl.storage_to_f64(wl.to_storage(want.astype(np.float32), dtype), dtype)
                assert np.array_equal(got, exp), "%s: %d mismatches" % (name, int((got != exp).sum()))
            else:
                err = oracle.max_normalised_error(got, want)
                assert err <= TOL[dtype], "%s: error %.3g" % (name, err)


def test_fused_maxpool_is_refused_where_no_tile_holds_the_image():
    L = B.lib()
    import ctypes
    for shape, dtype, kw in [(ConvShape(2, 32, 27, 27, 32, 3, 3, 1, 1), wl.F16, {}),            # 729 pixels, 3x3 window
                             (ConvShape(2, 32, 13, 13, 32, 5, 5, 1, 2), wl.F32, {}),            # fp32, 5x5 window
                             (ConvShape(2, 32, 13, 13, 32, 3, 3, 2, 1), wl.F16, {}),            # stride 2
                             (ConvShape(2, 3, 35, 35, 32, 11, 11, 4, 0), wl.F32, {})]:          # first layer in fp32
        d = B.desc_of(shape, dtype, maxpool=True, **kw)
        assert B.conv_variant_count(d) == 0
        assert L.conv_fwd(ctypes.byref(d), 256, 512, None, 1024, None) == B.CONV_ENOVARIANT


F32_POOL_SHAPES = [
    ConvShape(3, 64, 13, 13, 40, 3, 3, 1, 1),    # 13x13 -> 6x6, K ragged against the 16-row blocks
    ConvShape(2, 32, 14, 14, 64, 3, 3, 1, 1),    # 14x14 -> 6x6 on the 208-pixel tiles
    ConvShape(2, 32, 15, 15, 33, 3, 3, 1, 0),    # no padding: 13x13 -> 6x6
    ConvShape(2, 16, 12, 16, 16, 3, 3, 1, 1),    # 12x16 -> 5x7
]


@pytest.mark.parametrize("si", range(len(F32_POOL_SHAPES)))
def test_fused_maxpool_fp32_every_variant(si):
    torch = torch_mod()
    dtype = wl.F32
    shape = F32_POOL_SHAPES[si]
    PH, PW = (shape.OH - 3) // 2 + 1, (shape.OW - 3) // 2 + 1
    for ints, relu, use_bias in [(True, True, True), (True, False, False), (False, True, True)]:
        data = data_for(shape, dtype, 3500 + 10 * si, ints)
        conv = oracle.conv_fwd(data["in"].astype(np.float64), data["filt"].astype(np.float64),
                               data["bias"].astype(np.float64) if use_bias else None,
                               stride=shape.stride, pad=shape.pad, relu=relu)
        want = oracle.maxpool_fwd(conv, win=3, stride=2)
        d_in, d_filt = to_device(data["in"], dtype), to_device(data["filt"], dtype)
        d_bias = to_device(data["bias"], wl.F32) if use_bias else None
        fused = B.desc_of(shape, dtype, relu=relu, maxpool=True)
        plain = B.desc_of(shape, dtype, relu=relu)
        plain_names = [B.conv_variant_name(plain, i) for i in range(B.conv_variant_count(plain))]
        names = [B.conv_variant_name(fused, i) for i in range(B.conv_variant_count(fused))]
        assert names, "no variant pools %s" % (shape,)
        for vi, name in enumerate(names):
            say("  %s on %s ints=%s relu=%s bias=%s" % (name, shape, ints, relu, use_bias))
            out = run(fused, d_in, d_filt, d_bias, (shape.N, shape.K, PH, PW), dtype, vi)
            full = run(plain, d_in, d_filt, d_bias, shape.out_shape(), dtype, plain_names.index(name))
            seq = empty_out((shape.N, shape.K, PH, PW), dtype)
            B.maxpool_fwd(shape.N, shape.K, shape.OH, shape.OW, 3, 2, dtype, full, seq)
            torch.cuda.synchronize()
            got = out.cpu().numpy()
            assert np.array_equal(got.view(np.uint32), seq.cpu().numpy().view(np.uint32)), "%s: differs from conv + maxpool" % name
            assert np.all(np.isfinite(got)), "%s: unwritten elements" % name
            if ints:
                assert np.array_equal(got.astype(np.float64), want), "%s: mismatches" % name
            else:
                err = oracle.max_normalised_error(got.astype(np.float64), want)
                assert err <= TOL[dtype], "%s: error %.3g" % (name, err)


@pytest.mark.parametrize("relu", [True, False])
@pytest.mark.parametrize("dtype", [wl.F32, wl.F16])
def test_fused_maxpool_matches_the_sequence_on_nan_sums(dtype, relu):
    # a NaN in the input makes every convolution sum whose window holds it a NaN.  With the activation those become 0
    # before the pool in the two-call sequence; without it the NaN is the pooled result.  The fused call must agree.
    torch = torch_mod()
    shape = ConvShape(2, 32, 13, 13, 32, 3, 3, 1, 1)
    data = data_for(shape, dtype, 3900, False)
    x = wl.storage_to_f64(data["in"], dtype).astype(np.float32)
    x[0, 3, 6, 6] = np.nan
    x[1, 0, 0, 12] = np.nan
    data["in"] = wl.to_storage(x, dtype)
    PH, PW = (shape.OH - 3) // 2 + 1, (shape.OW - 3) // 2 + 1
    layouts = [(False, False)] if dtype == wl.F32 else [(False, False), (True, True), (True, False)]
    for in_nhwc, out_nhwc in layouts:
        d_in = to_device(nhwc(data["in"]) if in_nhwc else data["in"], dtype)
        d_filt = to_device(nhwc(data["filt"]) if in_nhwc else data["filt"], dtype)
        d_bias = to_device(data["bias"], wl.F32)
        kw = dict(relu=relu, in_nhwc=in_nhwc, out_nhwc=out_nhwc, filt_krsc=in_nhwc)
        fused, plain = B.desc_of(shape, dtype, maxpool=True, **kw), B.desc_of(shape, dtype, **kw)
        names = [B.conv_variant_name(fused, i) for i in range(B.conv_variant_count(fused))]
        plain_names = [B.conv_variant_name(plain, i) for i in range(B.conv_variant_count(plain))]
        assert names
        oshape = (shape.N, PH, PW, shape.K) if out_nhwc else (shape.N, shape.K, PH, PW)
        for vi, name in enumerate(names):
            say("  %s relu=%s in_nhwc=%s out_nhwc=%s" % (name, relu, in_nhwc, out_nhwc))
            out = run(fused, d_in, d_filt, d_bias, oshape, dtype, vi)
            full = run(plain, d_in, d_filt, d_bias,
                       (shape.N, shape.OH, shape.OW, shape.K) if out_nhwc else shape.out_shape(), dtype, plain_names.index(name))
            seq = empty_out(oshape, dtype)
            B.maxpool_fwd_layout(shape.N, shape.K, shape.OH, shape.OW, 3, 2, dtype, out_nhwc, out_nhwc, full, seq)
            torch.cuda.synchronize()
            got, want = to_host_f64(out, dtype), to_host_f64(seq, dtype)
            assert np.isnan(want).any() != relu, "the sequence's own NaN handling is not what this test assumes"
            assert np.array_equal(got, want, equal_nan=True), "%s: differs from conv + maxpool" % name


# First layers (3 channels, 11x11 stride 4 or 7x7 stride 2) whose pool is computed by the convolution kernel itself on
# tiles of 9x9 pooled outputs.
FIRST_POOL_SHAPES = [
    ConvShape(2, 3, 35, 35, 32, 11, 11, 4, 0),     # 7x7 -> 3x3: one partial tile per image
    ConvShape(2, 3, 91, 99, 96, 11, 11, 4, 2),     # 22x24 -> 10x11: 2x2 tiles, the last row and column of tiles partial; even OW
    ConvShape(1, 3, 227, 227, 40, 11, 11, 4, 0),   # the stack's first layer at one image: 55x55 -> 27x27 = 3x3 whole tiles; K ragged
    ConvShape(3, 3, 61, 57, 64, 7, 7, 2, 3),       # 31x29 -> 15x14, rows of odd length
    ConvShape(2, 3, 224, 224, 64, 7, 7, 2, 3),     # 112x112 -> 55x55: 7x7 tiles, rows of even length
    ConvShape(2, 3, 40, 44, 20, 7, 7, 2, 0),       # no padding, K below one channel block
]


@pytest.mark.parametrize("out_nhwc", [False, True])
@pytest.mark.parametrize("dtype", DT16)
@pytest.mark.parametrize("si", range(len(FIRST_POOL_SHAPES)))
def test_first_layer_fused_maxpool_every_variant(si, dtype, out_nhwc):
    torch = torch_mod()
    shape = FIRST_POOL_SHAPES[si]
    if out_nhwc and shape.K % 8:
        pytest.skip("channel-innermost pooled output needs K % 8 == 0")
    PH, PW = (shape.OH - 3) // 2 + 1, (shape.OW - 3) // 2 + 1
    oshape = (shape.N, PH, PW, shape.K) if out_nhwc else (shape.N, shape.K, PH, PW)
    for ints, relu, use_bias in [(True, True, True), (True, False, False), (False, True, True)]:
        data = data_for(shape, dtype, 4100 + 10 * si, ints)
        conv = oracle.conv_fwd(wl.storage_to_f64(data["in"], dtype), wl.storage_to_f64(data["filt"], dtype),
                               data["bias"].astype(np.float64) if use_bias else None,
                               stride=shape.stride, pad=shape.pad, relu=relu)
        want = oracle.maxpool_fwd(conv, win=3, stride=2)
        assert want.shape == (shape.N, shape.K, PH, PW)
        d_in, d_filt = to_device(data["in"], dtype), to_device(data["filt"], dtype)
        d_bias = to_device(data["bias"], wl.F32) if use_bias else None
        fused = B.desc_of(shape, dtype, relu=relu, out_nhwc=out_nhwc, maxpool=True)
        assert B.conv_out_shape(fused) == (PH, PW)
        names = [B.conv_variant_name(fused, i) for i in range(B.conv_variant_count(fused))]
        assert names and all(n.startswith("swinp_") for n in names), names
        # the two-call sequence: the same layer without the flag (any kernel), then the library's pool
        plain = B.desc_of(shape, dtype, relu=relu)
        full = empty_out(shape.out_shape(), dtype)
        B.conv_fwd(plain, d_in, d_filt, d_bias, full)
        seq = empty_out(oshape, dtype)
        B.maxpool_fwd_layout(shape.N, shape.K, shape.OH, shape.OW, 3, 2, dtype, False, out_nhwc, full, seq)
        torch.cuda.synchronize()
        seq = to_host_f64(seq, dtype)
        seq = nchw(seq) if out_nhwc else seq
        for vi, name in enumerate(names):
            say("  %s on %s dtype %d out_nhwc=%s ints=%s relu=%s bias=%s" % (name, shape, dtype, out_nhwc, ints, relu, use_bias))
            got = to_host_f64(run(fused, d_in, d_filt, d_bias, oshape, dtype, vi), dtype)
            got = nchw(got) if out_nhwc else got
            assert np.all(np.isfinite(got)), "%s: unwritten or overflowed elements" % name
            if ints:
                exp = wl.storage_to_f64(wl.to_storage(want.astype(np.float32), dtype), dtype)
                bad = np.argwhere(got != exp)
                assert bad.size == 0, "%s: %d mismatches, first at %s got %r want %r" % (
                    name, len(bad), tuple(bad[0]), got[tuple(bad[0])], exp[tuple(bad[0])])
                assert np.array_equal(got, seq), "%s: differs from conv + maxpool" % name
            else:
                err = oracle.max_normalised_error(got, want)
                assert err <= TOL[dtype], "%s: error %.3g" % (name, err)
                # against the library's own sequence: other kernels sum in another order, so within the tolerance only
                assert oracle.max_normalised_error(got, seq) <= 2 * TOL[dtype], name


@pytest.mark.parametrize("relu", [True, False])
def test_first_layer_fused_maxpool_on_nan_sums(relu):
    # as above for the first-layer kernel: with the activation a NaN sum pools as 0, without it the NaN is the result
    torch = torch_mod()
    dtype = wl.F16
    shape = ConvShape(2, 3, 91, 99, 32, 11, 11, 4, 2)
    data = data_for(shape, dtype, 4300, False)
    x = wl.storage_to_f64(data["in"], dtype).astype(np.float32)
    x[0, 1, 40, 40] = np.nan
    x[1, 2, 0, 98] = np.nan
    data["in"] = wl.to_storage(x, dtype)
    PH, PW = (shape.OH - 3) // 2 + 1, (shape.OW - 3) // 2 + 1
    d_in, d_filt, d_bias = to_device(data["in"], dtype), to_device(data["filt"], dtype), to_device(data["bias"], wl.F32)
    # every kernel of the layer itself puts its NaNs where the definition has them (none behind the activation)
    plain = B.desc_of(shape, dtype, relu=relu)
    conv_nan = np.isnan(oracle.conv_fwd(wl.storage_to_f64(data["in"], dtype), wl.storage_to_f64(data["filt"], dtype),
                                        data["bias"].astype(np.float64), stride=shape.stride, pad=shape.pad, relu=False))
    assert conv_nan.any()
    for vi in range(B.conv_variant_count(plain)):
        say("  %s relu=%s" % (B.conv_variant_name(plain, vi), relu))
        got = to_host_f64(run(plain, d_in, d_filt, d_bias, shape.out_shape(), dtype, vi), dtype)
        assert np.array_equal(np.isnan(got), conv_nan & (not relu)), B.conv_variant_name(plain, vi)
        assert np.all(np.isfinite(got[~conv_nan]))
    for out_nhwc in (False, True):
        oshape = (shape.N, PH, PW, shape.K) if out_nhwc else (shape.N, shape.K, PH, PW)
        fused = B.desc_of(shape, dtype, relu=relu, out_nhwc=out_nhwc, maxpool=True)
        full = empty_out(shape.out_shape(), dtype)
        B.conv_fwd(plain, d_in, d_filt, d_bias, full)
        seq = empty_out(oshape, dtype)
        B.maxpool_fwd_layout(shape.N, shape.K, shape.OH, shape.OW, 3, 2, dtype, False, out_nhwc, full, seq)
        torch.cuda.synchronize()
        want = to_host_f64(seq, dtype)
        assert np.isnan(want).any() != relu, "the sequence's own NaN handling is not what this test assumes"
        for vi in range(B.conv_variant_count(fused)):
            say("  %s relu=%s out_nhwc=%s" % (B.conv_variant_name(fused, vi), relu, out_nhwc))
            got = to_host_f64(run(fused, d_in, d_filt, d_bias, oshape, dtype, vi), dtype)
            assert np.array_equal(np.isnan(got), np.isnan(want)), "NaN results are not where the sequence has them"
            ok = ~np.isnan(want)
            assert oracle.max_normalised_error(got[ok], want[ok]) <= 2 * TOL[dtype]


@pytest.mark.parametrize("dtype", DT16)
def test_first_layer_fused_maxpool_random_shapes(dtype):
    # seeded random first layers (any image size from "one pooling window" up, any padding below the window, ragged K, both
    # output layouts): every pooled element against the oracle's convolution followed by its pool
    torch = torch_mod()
    rng = np.random.default_rng(4400 + dtype)
    for si in range(10):
        R, stride = [(11, 4), (7, 2)][int(rng.integers(0, 2))]
        lo = R + 2 * stride   # at least 3 convolution outputs per side: one pooling window
        shape = ConvShape(int(rng.choice([1, 2, 3])), 3, int(rng.integers(lo, 150)), int(rng.integers(lo, 150)),
                          int(rng.choice([8, 20, 32, 40, 64, 96, 100, 136])), R, R, stride, int(rng.integers(0, 4)))
        out_nhwc = bool(rng.integers(0, 2)) and shape.K % 8 == 0
        relu = bool(rng.integers(0, 4))
        use_bias = bool(rng.integers(0, 4))
        PH, PW = (shape.OH - 3) // 2 + 1, (shape.OW - 3) // 2 + 1
        oshape = (shape.N, PH, PW, shape.K) if out_nhwc else (shape.N, shape.K, PH, PW)
        for ints in (True, False):
            data = data_for(shape, dtype, 4500 + 10 * si, ints)
            conv = oracle.conv_fwd(wl.storage_to_f64(data["in"], dtype), wl.storage_to_f64(data["filt"], dtype),
                                   data["bias"].astype(np.float64) if use_bias else None,
                                   stride=shape.stride, pad=shape.pad, relu=relu)
            want = oracle.maxpool_fwd(conv, win=3, stride=2)
            d_in, d_filt = to_device(data["in"], dtype), to_device(data["filt"], dtype)
            d_bias = to_device(data["bias"], wl.F32) if use_bias else None
            fused = B.desc_of(shape, dtype, relu=relu, out_nhwc=out_nhwc, maxpool=True)
            names = [B.conv_variant_name(fused, i) for i in range(B.conv_variant_count(fused))]
            assert names, "no variant pools %s" % (shape,)
            for vi, name in enumerate(names):
                say("  %s on %s dtype %d out_nhwc=%s ints=%s relu=%s bias=%s" % (name, shape, dtype, out_nhwc, ints, relu, use_bias))
                got = to_host_f64(run(fused, d_in, d_filt, d_bias, oshape, dtype, vi), dtype)
                got = nchw(got) if out_nhwc else got
                assert np.all(np.isfinite(got)), "%s: unwritten or overflowed elements" % name
                if ints:
                    exp = wl.storage_to_f64(wl.to_storage(want.astype(np.float32), dtype), dtype)
                    bad = np.argwhere(got != exp)
                    assert bad.size == 0, "%s on %s: %d mismatches, first at %s got %r want %r" % (
                        name, shape, len(bad), tuple(bad[0]), got[tuple(bad[0])], exp[tuple(bad[0])])
                else:
                    err = oracle.max_normalised_error(got, want)
                    assert err <= TOL[dtype], "%s on %s: error %.3g" % (name, shape, err)
