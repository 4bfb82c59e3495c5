"""GPU parity near the library's size limits: tensors of 3.3 to 3.9 GB (byte offsets that no longer fit a signed
32-bit integer; the documented limit is 4 GiB and 2^31 elements per tensor), checked against the CPU oracle on bands
of output rows at the lowest and the highest addresses.

Small-integer data: every variant must agree with the oracle bit for bit.
"""
import numpy as np
import pytest

import oracle
from paper_1611_06945_amd import binding as B
from paper_1611_06945_amd import workloads as wl
from paper_1611_06945_amd.workloads import ConvShape

from gpu_util import to_device, torch_mod
from test_gpu_parity import say

pytestmark = pytest.mark.gpu


def oracle_rows(x_img, filt, bias, shape, a, b, relu):
    """Output rows [a, b) of one image ([C][H][W] in float64), from the band of input rows they read."""
    top, bot = a * shape.stride - shape.pad, (b - 1) * shape.stride - shape.pad + shape.R
    band = np.zeros((1, shape.C, bot - top, shape.W + 2 * shape.pad))
    lo, hi = max(top, 0), min(bot, shape.H)
    band[0, :, lo - top:hi - top, shape.pad:shape.pad + shape.W] = x_img[:, lo:hi, :]
    return oracle.conv_fwd(band, filt, bias, stride=shape.stride, pad=0, relu=relu)[0]


LARGE = [
    # input of 3.90 GB (the limit is 4 GiB per tensor), small output: window origins at byte offsets up to nearly 2^32
    (ConvShape(3, 40, 2800, 2900, 8, 3, 3, 7, 1), wl.F32),
    # output of 3.46 GB from a small input: store offsets beyond 2^31
    (ConvShape(3, 8, 1500, 1500, 128, 1, 1, 1, 0), wl.F32),
    # 16-bit input of 3.32 GB (1.66e9 elements; the limit is 2^31 elements)
    (ConvShape(3, 24, 4800, 4800, 8, 5, 5, 9, 2), wl.F16),
    (ConvShape(3, 24, 4800, 4800, 8, 5, 5, 9, 2), wl.BF16),
    # inputs just below 1 GiB, the limit of the kernels that fold window offsets into 32-bit sums (precomputed-offset
    # implicit GEMM, Winograd, channel-innermost)
    (ConvShape(4, 64, 1020, 1020, 32, 3, 3, 1, 1), wl.F32),
    (ConvShape(8, 64, 1020, 1020, 32, 3, 3, 1, 1), wl.F16),
    (ConvShape(8, 64, 1020, 1020, 32, 3, 3, 1, 1), wl.BF16),
    # many small images, 1.53 GB in all: the Winograd kernels' domain (input below 2 GiB including their look-ahead)
    (ConvShape(1900, 64, 56, 56, 32, 3, 3, 1, 1), wl.F32),
]


@pytest.mark.parametrize("ci", range(len(LARGE)))
def test_tensors_close_to_the_size_limits(ci):
    shape, dtype = LARGE[ci]
    run_large(ci, shape, dtype, False)


@pytest.mark.parametrize("ci", [5, 6])
def test_channel_innermost_tensors_close_to_the_size_limit(ci):
    shape, dtype = LARGE[ci]
    run_large(ci, shape, dtype, True)


def run_large(ci, shape, dtype, nhwc):
    torch = torch_mod()
    relu = True
    tdt = {wl.F32: torch.float32, wl.F16: torch.float16, wl.BF16: torch.bfloat16}[dtype]
    d_in = torch.empty(shape.in_shape(), dtype=tdt, device="cuda")
    first = last = None
    for n in range(shape.N):
        img = wl.to_storage(wl.draw(("int", -3, 3), (shape.C, shape.H, shape.W), 7000 + 10 * ci + n), dtype)
        d_in[n].copy_(to_device(img, dtype))
        if n == 0:
            first = img
        if n == shape.N - 1:
            last = img
    filt = wl.to_storage(wl.draw(("int", -2, 2), shape.filt_shape(), 7100 + ci), dtype)
    bias = wl.draw(("int", -4, 4), (shape.K,), 7200 + ci)
    d_filt, d_bias = to_device(filt, dtype), to_device(bias, wl.F32)
    if nhwc:  # the same tensors stored channel-innermost (plain device-side permutations: test plumbing)
        d_in = d_in.permute(0, 2, 3, 1).contiguous()
        d_filt = d_filt.permute(0, 2, 3, 1).contiguous()
    f64, b64 = wl.storage_to_f64(filt, dtype), bias.astype(np.float64)

    OH = shape.OH
    bands = [(0, 0, min(3, OH), first), (0, OH // 2, min(OH // 2 + 2, OH), first),
             (shape.N - 1, max(OH - 3, 0), OH, last)]
    want = []
    for (n, a, b, img) in bands:
        ref = oracle_rows(wl.storage_to_f64(img, dtype), f64, b64, shape, a, b, relu)
        want.append(wl.storage_to_f64(wl.to_storage(ref.astype(np.float32), dtype), dtype))

    desc = B.desc_of(shape, dtype, relu=relu, in_nhwc=nhwc, out_nhwc=nhwc, filt_krsc=nhwc)
    names = [B.conv_variant_name(desc, i) for i in range(B.conv_variant_count(desc))]
    assert names, "no variant for %s" % (shape,)
    ws = torch.empty(max(256, B.conv_workspace_bytes(desc)), dtype=torch.uint8, device="cuda")
    oshape = (shape.N, shape.OH, shape.OW, shape.K) if nhwc else shape.out_shape()
    out = torch.empty(oshape, dtype=tdt, device="cuda")
    for vi in list(range(len(names))) + [-1]:
        name = names[vi] if vi >= 0 else "default (%s)" % B.conv_variant_name(desc, -1)
        say("  %s on %s dtype %d" % (name, shape, dtype))
        out.fill_(float("nan"))  # an element no kernel writes stays NaN
        B.conv_force_variant(desc, vi)
        try:
            B.conv_fwd_ws(desc, d_in, d_filt, d_bias, out, ws, ws.numel())
            torch.cuda.synchronize()
        finally:
            B.conv_force_variant(desc, -1)
        assert not bool(torch.isnan(out).any()), "%s: unwritten output elements" % name
        for (n, a, b, _), exp in zip(bands, want):
            rows = out[n, a:b, :, :].permute(2, 0, 1) if nhwc else out[n, :, a:b, :]
            if dtype == wl.BF16:
                got = wl.storage_to_f64(rows.contiguous().view(torch.int16).cpu().numpy().view(np.uint16), dtype)
            else:
                got = rows.contiguous().cpu().numpy().astype(np.float64)
            bad = np.argwhere(got != exp)
            assert bad.size == 0, "%s image %d rows %d..%d: %d mismatches, first at %s got %r want %r" % (
                name, n, a, b, len(bad), tuple(bad[0]), got[tuple(bad[0])], exp[tuple(bad[0])])
