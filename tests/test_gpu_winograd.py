"""GPU parity of the Winograd F(2x2, 3x3) variants (fp32, 3x3 stride-1 layers) against the CPU oracle.

The variants compute the same convolution as the direct kernels through a different arithmetic (filter, input and
output transforms around 16 small matrix products), so the oracle is the plain definition itself.  On small-integer data
every product and sum of the transformed values is exact (the filter transform only halves), hence bit-exact results;
on random data the fp32 tolerance of the direct kernels applies unchanged (1e-5 max normalised error).
"""
import numpy as np
import pytest

from paper_1611_06945_amd import binding as B
from paper_1611_06945_amd import workloads as wl
from paper_1611_06945_amd.workloads import ConvShape

from gpu_util import TOL, DeviceCase, empty_out, to_host_f64, torch_mod
from test_gpu_parity import assert_bit_exact, int_case, random_case, say

pytestmark = pytest.mark.gpu

# (shape, why)
WINO_SHAPES = [
    (ConvShape(3, 16, 13, 13, 40, 3, 3, 1, 1), "odd image: the last tile row and column are half outside; K ragged"),
    (ConvShape(2, 8, 14, 14, 33, 3, 3, 1, 1), "even image, one step of 8 channels, K ragged"),
    (ConvShape(1, 24, 7, 9, 20, 3, 3, 1, 0), "no padding, non-square, 5x7 outputs"),
    (ConvShape(5, 8, 5, 6, 16, 3, 3, 1, 1), "tiny images: one workgroup's tiles span several images"),
    (ConvShape(2, 40, 28, 28, 50, 3, 3, 1, 1), "28x28: several workgroups per image, five steps"),
    (ConvShape(1, 16, 56, 56, 16, 3, 3, 1, 1), "56x56: two staging slots per thread needed by the wider tiles"),
    (ConvShape(1, 8, 3, 3, 5, 3, 3, 1, 0), "single output pixel per image and channel"),
    (ConvShape(7, 32, 4, 4, 64, 3, 3, 1, 1), "4x4 images, four tiles each"),
]


def wino_variants(case):
    return [(i, n) for i, n in enumerate(case.variant_names()) if n.startswith("wino_")]


@pytest.mark.parametrize("wi", range(len(WINO_SHAPES)))
def test_every_winograd_variant(wi):
    shape, why = WINO_SHAPES[wi]
    icase = int_case(shape, wl.F32, 900 + wi)
    rcase = random_case(shape, wl.F32, 950 + wi)
    variants = wino_variants(icase)
    assert variants, "no Winograd variant for %s" % (shape,)
    for vi, name in variants:
        say("  %s on %s (%s)" % (name, shape, why))
        assert_bit_exact(icase, icase.run(variant=vi), name)
        err = rcase.error(rcase.run(variant=vi))
        assert err <= TOL[wl.F32], "%s: error %.3g" % (name, err)


def test_without_bias_and_activation():
    shape = ConvShape(2, 16, 13, 13, 40, 3, 3, 1, 1)
    case = random_case(shape, wl.F32, 970, relu=False, use_bias=False)
    for vi, name in wino_variants(case):
        err = case.error(case.run(variant=vi))
        assert err <= TOL[wl.F32], "%s: error %.3g" % (name, err)
        assert np.any(case.ref() < 0)  # the test would not see a stray activation otherwise


def test_benchmark_shape_every_output():
    """Configuration 4 at batch 5 (the paper's batch), every output element, the variants with the shortest measured time."""
    w = wl.config4(5, wl.F32)
    case = DeviceCase(w.shape, w.dtype, w.generate(), relu=True, use_bias=True)
    variants = wino_variants(case)
    assert variants
    for vi, name in variants[:4]:
        err = case.error(case.run(variant=vi))
        say("  %s on %s: max normalised error %.3g" % (name, w.name, err))
        assert err <= TOL[wl.F32], "%s: error %.3g" % (name, err)


def test_runs_are_bit_reproducible():
    shape = ConvShape(3, 32, 13, 13, 48, 3, 3, 1, 1)
    case = random_case(shape, wl.F32, 980)
    for vi, name in wino_variants(case)[:3]:
        a = case.run(variant=vi).cpu().numpy()
        b = case.run(variant=vi).cpu().numpy()
        assert np.array_equal(a, b), name


def test_workspace_is_required_and_sized_for_the_transformed_filters():
    shape = ConvShape(2, 16, 13, 13, 38, 3, 3, 1, 1)
    case = random_case(shape, wl.F32, 990)
    vi, name = wino_variants(case)[0]
    kp = (shape.K + 3) // 4 * 4
    assert B.conv_variant_workspace(case.desc, vi) == 16 * kp * shape.C * 4
    assert B.conv_workspace_bytes(case.desc) >= 16 * kp * shape.C * 4
    B.conv_force_variant(case.desc, vi)
    try:
        out = empty_out(shape.out_shape(), wl.F32)
        with pytest.raises(B.ConvError) as e:
            B.conv_fwd(case.desc, case.d_in, case.d_filt, case.d_bias, out)
        assert e.value.status == B.CONV_EWORKSPACE
    finally:
        B.conv_force_variant(case.desc, -1)


def test_not_offered_outside_its_domain():
    for shape, dtype in [
        (ConvShape(2, 16, 13, 13, 40, 3, 3, 1, 1), wl.F16),   # 16-bit storage: the transforms would dominate
        (ConvShape(2, 16, 13, 13, 40, 3, 3, 2, 1), wl.F32),   # stride 2
        (ConvShape(2, 16, 13, 13, 40, 5, 5, 1, 2), wl.F32),   # 5x5
        (ConvShape(2, 12, 13, 13, 40, 3, 3, 1, 1), wl.F32),   # channels not a multiple of the step
        (ConvShape(2, 16, 13, 13, 40, 3, 3, 1, 2), wl.F32),   # padding wider than the window overlap
    ]:
        desc = B.desc_of(shape, dtype, relu=True)
        names = [B.conv_variant_name(desc, i) for i in range(B.conv_variant_count(desc))]
        assert names and not any(n.startswith("wino_") for n in names), (shape, dtype)


def test_filters_handed_over_in_the_winograd_domain():
    """conv_transform_filters + CONV_FLAG_FILT_WINOGRAD: same bits as the in-call transform, no workspace needed."""
    torch = torch_mod()
    for shape in [ConvShape(3, 16, 13, 13, 38, 3, 3, 1, 1), ConvShape(2, 24, 14, 10, 64, 3, 3, 1, 0)]:
        case = random_case(shape, wl.F32, 1000)
        pre = B.desc_of(shape, wl.F32, relu=True, filt_winograd=True)
        nbytes = B.conv_transformed_filter_bytes(case.desc)
        assert nbytes == B.conv_transformed_filter_bytes(pre) > 0
        # poisoned: rows K..K' of the format are never written and must not matter
        u = torch.full((nbytes // 4,), float("nan"), dtype=torch.float32, device="cuda")
        B.conv_transform_filters(case.desc, case.d_filt, u)
        names_pre = [B.conv_variant_name(pre, i) for i in range(B.conv_variant_count(pre))]
        assert names_pre
        plain_names = case.variant_names()
        for vi, name in enumerate(names_pre):
            say("  %s with pre-transformed filters on %s" % (name, shape))
            out = empty_out(shape.out_shape(), wl.F32)
            B.conv_force_variant(pre, vi)
            try:
                B.conv_fwd(pre, case.d_in, u, case.d_bias, out)   # no workspace
                torch.cuda.synchronize()
            finally:
                B.conv_force_variant(pre, -1)
            ref = case.run(variant=plain_names.index(name))       # the same variant transforming in the call
            assert np.array_equal(out.cpu().numpy(), ref.cpu().numpy()), name
            assert case.error(out) <= TOL[wl.F32]


def test_variants_that_transform_filters_in_the_kernel_need_no_workspace():
    """The "_ff" variants read the filters as they are: conv_fwd (no workspace) can run them, and once the layer has been
    autotuned that entry point uses the fastest variant that needs no workspace."""
    torch = torch_mod()
    shape = ConvShape(4, 32, 13, 13, 96, 3, 3, 1, 1)
    case = random_case(shape, wl.F32, 1010)
    ff = [(i, n) for i, n in wino_variants(case) if n.endswith("_ff")]
    assert ff
    for vi, name in ff:
        assert B.conv_variant_workspace(case.desc, vi) == 0
        err = case.error(case.run(variant=vi, with_ws=False))
        say("  %s through conv_fwd: max normalised error %.3g" % (name, err))
        assert err <= TOL[wl.F32], "%s: error %.3g" % (name, err)
    ws = case.workspace()
    out = empty_out(shape.out_shape(), wl.F32)
    B.conv_autotune(case.desc, case.d_in, case.d_filt, case.d_bias, out, ws, ws.numel())
    n = B.conv_variant_count(case.desc)
    times = {B.conv_variant_name(case.desc, i): B.conv_variant_time_us(case.desc, i) for i in range(n)}
    no_ws = {B.conv_variant_name(case.desc, i) for i in range(n) if B.conv_variant_workspace(case.desc, i) == 0}
    fastest_no_ws = min(no_ws, key=lambda nm: times[nm])
    # conv_fwd has no workspace to offer: the name reported for it is the fastest variant that needs none
    out2 = empty_out(shape.out_shape(), wl.F32)
    B.conv_fwd(case.desc, case.d_in, case.d_filt, case.d_bias, out2)
    torch.cuda.synchronize()
    assert case.error(out2) <= TOL[wl.F32]
    say("  fastest without workspace: %s (%.1f us)" % (fastest_no_ws, times[fastest_no_ws]))
    assert B.conv_variant_name(case.desc, -2) == fastest_no_ws   # idx -2: what conv_fwd runs
    B.conv_cache_clear()
