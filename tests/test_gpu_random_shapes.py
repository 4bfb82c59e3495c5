"""GPU parity on seeded random problem shapes: every variant the library offers for a shape, against the CPU oracle.

The shapes are drawn from the ranges of the networks' layers (Appendix A: windows 1 to 11, strides 1 to 4, 3 to
a few hundred channels) scaled down so that the oracle finishes at once; none of them is chosen to suit a tile.
"""
import numpy as np
import pytest

import oracle

from paper_1611_06945_amd import workloads as wl
from paper_1611_06945_amd.workloads import ConvShape

from gpu_util import TOL
from test_gpu_parity import assert_bit_exact, int_case, random_case, say

pytestmark = pytest.mark.gpu

DTYPES = [wl.F32, wl.F16, wl.BF16]
GROUPS = 16
SHAPES_PER_GROUP = 6


def draw_shape(rng):
    """One random convolution; rejects windows larger than the padded image and work beyond ~40 MFLOP."""
    while True:
        R = int(rng.choice([1, 1, 3, 3, 3, 5, 5, 7, 11]))
        S = R if rng.random() < 0.85 else int(rng.choice([1, 3, 5]))
        stride = int(rng.choice([1, 1, 1, 2, 2, 4])) if R > 1 else int(rng.choice([1, 1, 1, 2]))
        pad = int(rng.choice([0, R // 2, R // 2, min(R // 2 + 1, 3)]))
        C = int(rng.choice([1, 3, 3, 4, 8, 16, 16, 24, 32, 32, 48, 64, 96, 100]))
        K = int(rng.choice([1, 4, 8, 16, 20, 32, 33, 48, 64, 96, 100, 130]))
        H = int(rng.integers(1, 41))
        W = int(rng.integers(1, 41))
        N = int(rng.choice([1, 1, 2, 3, 5]))
        if H + 2 * pad < R or W + 2 * pad < S:
            continue
        shape = ConvShape(N, C, H, W, K, R, S, stride, pad)
        if shape.flops > 4e7:
            continue
        return shape


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("group", range(GROUPS))
def test_random_shapes_every_variant(group, dtype):
    rng = np.random.default_rng(9000 + group)
    for si in range(SHAPES_PER_GROUP):
        shape = draw_shape(rng)
        relu = bool(rng.integers(0, 2))
        use_bias = bool(rng.integers(0, 4))
        seed = 9100 + 100 * group + si
        icase = int_case(shape, dtype, seed, relu=relu, use_bias=use_bias)
        rcase = random_case(shape, dtype, seed + 50, relu=relu, use_bias=use_bias)
        names = icase.variant_names()
        assert names, "no variant for %s" % (shape,)
        say("  %s dtype %d relu=%s bias=%s: %d variants" % (shape, dtype, relu, use_bias, len(names)))
        for vi, name in enumerate(names):
            assert_bit_exact(icase, icase.run(variant=vi), "%s on %s" % (name, shape))
            err = rcase.error(rcase.run(variant=vi))
            assert err <= TOL[dtype], "%s on %s: error %.3g" % (name, shape, err)
        # the default selection, with and without a workspace
        assert_bit_exact(icase, icase.run(variant=-1, with_ws=True), "default on %s" % (shape,))
        assert_bit_exact(icase, icase.run(variant=-1, with_ws=False), "default without workspace on %s" % (shape,))


def draw_family_shape(rng, family):
    """A random shape inside the domain of one of the specialised kernel families."""
    while True:
        N = int(rng.choice([1, 2, 3, 5]))
        if family == "first_layer":  # few input channels, big strided window
            R, stride = [(11, 4), (7, 2)][int(rng.integers(0, 2))]
            # wide images: the 16-bit strided-window kernels want 128 consecutive outputs within a few output rows
            shape = ConvShape(N, 3, int(rng.integers(R, 60)), int(rng.integers(100, 255)),
                              int(rng.choice([4, 8, 20, 32, 64, 96, 100])), R, R, stride, int(rng.integers(0, 4)))
        elif family == "window3":  # 3x3 stride 1 over whole 16-channel chunks: window kernels and Winograd
            shape = ConvShape(N, 16 * int(rng.integers(1, 7)), int(rng.integers(3, 31)), int(rng.integers(3, 31)),
                              int(rng.choice([8, 16, 33, 48, 64, 100, 130])), 3, 3, 1, int(rng.integers(0, 3)))
        elif family == "window5":
            shape = ConvShape(N, 16 * int(rng.integers(1, 4)), int(rng.integers(5, 31)), int(rng.integers(5, 31)),
                              int(rng.choice([8, 32, 33, 64, 100])), 5, 5, 1, int(rng.integers(0, 3)))
        elif family == "pointwise":
            shape = ConvShape(N, int(rng.choice([16, 32, 40, 64, 128, 200])), int(rng.integers(1, 31)),
                              int(rng.integers(1, 31)), int(rng.choice([8, 16, 33, 64, 100, 130])), 1, 1, 1, 0)
        else:  # fully connected: the window covers the image
            H, W = int(rng.integers(1, 8)), int(rng.integers(1, 8))
            shape = ConvShape(N, int(rng.choice([8, 16, 64, 100, 256, 1032])), H, W,
                              int(rng.choice([10, 33, 64, 130, 500])), H, W, 1, 0)
        if shape.flops <= 1e8:
            return shape


FAMILIES = ["first_layer", "window3", "window5", "pointwise", "fully_connected"]


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("family", FAMILIES)
def test_random_shapes_in_the_domains_of_the_specialised_kernels(family, dtype):
    rng = np.random.default_rng(9500 + FAMILIES.index(family))
    for si in range(8):
        shape = draw_family_shape(rng, family)
        relu = bool(rng.integers(0, 2))
        use_bias = bool(rng.integers(0, 4))
        seed = 9600 + 100 * FAMILIES.index(family) + si
        icase = int_case(shape, dtype, seed, relu=relu, use_bias=use_bias)
        rcase = random_case(shape, dtype, seed + 50, relu=relu, use_bias=use_bias)
        names = icase.variant_names()
        assert names, "no variant for %s" % (shape,)
        say("  %s: %s dtype %d relu=%s bias=%s: %d variants" % (family, shape, dtype, relu, use_bias, len(names)))
        for vi, name in enumerate(names):
            assert_bit_exact(icase, icase.run(variant=vi), "%s on %s" % (name, shape))
            err = rcase.error(rcase.run(variant=vi))
            assert err <= TOL[dtype], "%s on %s: error %.3g" % (name, shape, err)


@pytest.mark.parametrize("dtype", [wl.F16, wl.BF16])
@pytest.mark.parametrize("group", range(4))
def test_random_shapes_channel_innermost(group, dtype):
    from test_gpu_nhwc import NhwcCase

    rng = np.random.default_rng(9800 + group)
    done = 0
    while done < 6:
        shape = draw_shape(rng) if done % 2 else draw_family_shape(rng, ["window3", "window5"][done // 2 % 2])
        out_nhwc = bool(rng.integers(0, 2))
        relu = bool(rng.integers(0, 2))
        if shape.C % 8 or (out_nhwc and shape.K % 8):
            continue  # the channel-innermost kernels move whole 16-byte channel vectors, in and out
        seed = 9900 + 100 * group + done
        done += 1
        icase = NhwcCase(shape, dtype, wl.small_int_case(shape, dtype, seed), out_nhwc, relu=relu)
        rdata = {
            "in": wl.to_storage(wl.draw(("uniform", -1.0, 1.0), shape.in_shape(), seed + 50), dtype),
            "filt": wl.to_storage(wl.draw(("normal", wl.he_sigma(shape)), shape.filt_shape(), seed + 51), dtype),
            "bias": wl.draw(("uniform", -0.1, 0.1), (shape.K,), seed + 52),
        }
        rcase = NhwcCase(shape, dtype, rdata, out_nhwc, relu=relu)
        names = icase.names()
        assert names, "no channel-innermost variant for %s" % (shape,)
        say("  nhwc: %s dtype %d out_nhwc=%s relu=%s: %d variants" % (shape, dtype, out_nhwc, relu, len(names)))
        want = wl.storage_to_f64(wl.to_storage(icase.ref.astype(np.float32), dtype), dtype)
        for vi, name in enumerate(names):
            got = icase.run(variant=vi)
            assert np.array_equal(got, want), "%s on %s: %d mismatches" % (name, shape, int((got != want).sum()))
            rgot = rcase.run(variant=vi)
            assert np.all(np.isfinite(rgot)), "%s on %s: unwritten or overflowed elements" % (name, shape)
            err = oracle.max_normalised_error(rgot, rcase.ref)
            assert err <= TOL[dtype], "%s on %s: error %.3g" % (name, shape, err)
