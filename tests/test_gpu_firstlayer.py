"""GPU parity of the strided window variants for first layers (3 input channels, 11x11 stride 4 and 7x7 stride 2,
fp16 / bf16 storage) against the CPU oracle, through the C ABI.

The variants stage the input rows of a tile in LDS and pad every filter row to a multiple of 4 taps; the cases below
cover what that layout can get wrong: rows of odd length (a staged row starts at any 2-byte alignment in memory),
tiles that span several output rows and end inside one, the last tile of an image, images smaller than a tile,
zero padding on all four sides, ragged channel counts, and non-finite inputs next to a window (the padding taps must
not let them through).
"""
import numpy as np
import pytest

import oracle

from paper_1611_06945_amd import binding as B
from paper_1611_06945_amd import workloads as wl
from paper_1611_06945_amd.workloads import ConvShape

from gpu_util import TOL, DeviceCase, empty_out, to_host_f64, torch_mod
from test_gpu_parity import assert_bit_exact, int_case, random_case, say

pytestmark = pytest.mark.gpu

# (shape, why)
SWIN_SHAPES = [
    (ConvShape(2, 3, 227, 227, 96, 11, 11, 4, 0), "the benchmark's first layer: rows of 55 outputs, 23.6 tiles per image"),
    (ConvShape(1, 3, 224, 224, 96, 11, 11, 4, 0), "rows of 54 outputs, even row length"),
    (ConvShape(3, 3, 23, 63, 40, 11, 11, 4, 0), "image smaller than a tile (56 outputs), ragged channel count"),
    (ConvShape(2, 3, 19, 75, 64, 11, 11, 4, 2), "zero padding 2 on every side"),
    (ConvShape(1, 3, 227, 227, 20, 11, 11, 4, 0), "fewer channels than the smallest tile"),
    (ConvShape(2, 3, 11, 130, 64, 7, 7, 2, 3), "7x7 stride 2 with padding 3, rows of 65 outputs"),
    (ConvShape(1, 3, 224, 224, 64, 7, 7, 2, 3), "7x7 stride 2: the 224x224 first layer, rows of 112 outputs"),
    (ConvShape(2, 3, 40, 200, 32, 7, 7, 2, 0), "7x7 stride 2 without padding, rows of 97 outputs"),
]


def swin_variants(case):
    return [(i, n) for i, n in enumerate(case.variant_names()) if n.startswith("swin_")]


@pytest.mark.parametrize("dtype", [wl.F16, wl.BF16])
@pytest.mark.parametrize("wi", range(len(SWIN_SHAPES)))
def test_every_strided_window_variant(wi, dtype):
    shape, why = SWIN_SHAPES[wi]
    icase = int_case(shape, dtype, 1100 + wi)
    rcase = random_case(shape, dtype, 1150 + wi)
    variants = swin_variants(icase)
    assert variants, "no strided window variant for %s" % (shape,)
    for vi, name in variants:
        say("  %s on %s (%s)" % (name, shape, why))
        assert_bit_exact(icase, icase.run(variant=vi), name)
        err = rcase.error(rcase.run(variant=vi))
        assert err <= TOL[dtype], "%s: error %.3g" % (name, err)


def test_without_bias_and_activation():
    shape = ConvShape(2, 3, 59, 227, 96, 11, 11, 4, 0)
    case = random_case(shape, wl.F16, 1170, relu=False, use_bias=False)
    variants = swin_variants(case)
    assert variants
    for vi, name in variants:
        err = case.error(case.run(variant=vi))
        assert err <= TOL[wl.F16], "%s: error %.3g" % (name, err)
        assert np.any(case.ref() < 0)


def test_benchmark_first_layer_every_output():
    """Configuration 5's first layer at batch 5, every output element, every variant."""
    shape = ConvShape(5, 3, 227, 227, 96, 11, 11, 4, 0)
    case = random_case(shape, wl.F16, 1180)
    variants = swin_variants(case)
    assert variants
    for vi, name in variants:
        err = case.error(case.run(variant=vi))
        say("  %s on %s: max normalised error %.3g" % (name, shape, err))
        assert err <= TOL[wl.F16], "%s: error %.3g" % (name, err)


def test_non_finite_input_stays_inside_its_windows():
    """An infinite input value must reach the outputs whose window holds it and no other: the taps that pad a filter
    row to a multiple of 4 read the neighbouring window's first column, and are masked."""
    shape = ConvShape(1, 3, 23, 227, 32, 11, 11, 4, 0)
    base = random_case(shape, wl.F16, 1190, relu=False)
    data = {k: v.copy() for k, v in base.data.items()}
    inf16 = wl.to_storage(np.array([np.inf], dtype=np.float32), wl.F16)[0]
    for col in (11, 12 + 4 * 20, 226):   # right after window 0, inside the row, the last column
        data["in"][0, 1, 5, col] = inf16
    case = DeviceCase(shape, wl.F16, data, relu=False, use_bias=True)
    ref = case.ref()
    clean = np.isfinite(ref)
    assert 0 < clean.sum() < clean.size
    for vi, name in swin_variants(case):
        got = to_host_f64(case.run(variant=vi), wl.F16)
        assert np.all(np.isfinite(got[clean])), name
        assert np.all(~np.isfinite(got[~clean])), name
        err = np.max(np.abs(got[clean] - ref[clean])) / np.max(np.abs(ref[clean]))
        assert err <= TOL[wl.F16], "%s: error %.3g" % (name, err)


@pytest.mark.parametrize("dtype", [wl.F16, wl.BF16])
def test_channel_innermost_output_from_planar_input(dtype):
    """CONV_FLAG_OUT_NHWC alone: the same kernels write [N][OH][OW][K] (what a channel-innermost second layer or pool
    consumes) from planar input and filters; compared with the oracle after transposing back, bit-exact on integers."""
    torch = torch_mod()
    for si, shape in enumerate([ConvShape(2, 3, 227, 227, 96, 11, 11, 4, 0), ConvShape(3, 3, 23, 63, 40, 11, 11, 4, 0),
                                ConvShape(2, 3, 11, 130, 64, 7, 7, 2, 3)]):
        icase = int_case(shape, dtype, 1200 + si)
        rcase = random_case(shape, dtype, 1210 + si)
        desc = B.desc_of(shape, dtype, relu=True, out_nhwc=True)
        names = [B.conv_variant_name(desc, i) for i in range(B.conv_variant_count(desc))]
        assert names and all(n.startswith("swin_") for n in names), names
        exp_int = wl.storage_to_f64(wl.to_storage(icase.ref().astype(np.float32), dtype), dtype)
        for vi, name in enumerate(names):
            say("  %s writing channel-innermost on %s" % (name, shape))
            for case, exact in ((icase, True), (rcase, False)):
                out = empty_out((shape.N, shape.OH, shape.OW, shape.K), dtype)
                B.conv_force_variant(desc, vi)
                try:
                    B.conv_fwd(desc, case.d_in, case.d_filt, case.d_bias, out)
                    torch.cuda.synchronize()
                finally:
                    B.conv_force_variant(desc, -1)
                got = np.ascontiguousarray(np.transpose(to_host_f64(out, dtype), (0, 3, 1, 2)))
                assert np.all(np.isfinite(got)), name
                if exact:
                    assert np.array_equal(got, exp_int), name
                else:
                    err = oracle.max_normalised_error(got, case.ref())
                    assert err <= TOL[dtype], "%s: error %.3g" % (name, err)
    # a channel count that is no multiple of 4 has no such kernel
    assert B.conv_variant_count(B.desc_of(ConvShape(1, 3, 227, 227, 30, 11, 11, 4, 0), dtype, out_nhwc=True)) == 0


def test_not_offered_outside_its_domain():
    for shape, dtype in [
        (ConvShape(2, 3, 227, 227, 96, 11, 11, 4, 0), wl.F32),   # fp32 storage
        (ConvShape(2, 4, 227, 227, 96, 11, 11, 4, 0), wl.F16),   # another channel count
        (ConvShape(2, 3, 227, 227, 96, 11, 11, 2, 0), wl.F16),   # another stride
        (ConvShape(2, 3, 63, 63, 96, 11, 11, 4, 0), wl.F16),     # rows of 14 outputs: a tile would span 10 output rows
        (ConvShape(1, 3, 227, 600, 96, 11, 11, 4, 0), wl.F16),   # rows longer than the staging covers
    ]:
        desc = B.desc_of(shape, dtype, relu=True)
        names = [B.conv_variant_name(desc, i) for i in range(B.conv_variant_count(desc))]
        assert names and not any(n.startswith("swin_") for n in names), (shape, dtype)
