"""GPU parity of the channel-innermost path: the explicit format conversions, the layout-aware max-pool and the
NHWC/KRSC convolution kernels (fp16/bf16), element by element against the CPU oracle.  The oracle only knows the
paper's layouts ([N][C][H][W], [K][C][R][S]); host-side numpy transposes carry data between the two worlds."""
import numpy as np
import pytest

import oracle
from paper_1611_06945_amd import binding as B
from paper_1611_06945_amd import workloads as wl
from paper_1611_06945_amd.workloads import ConvShape

from gpu_util import TOL, empty_out, to_device, to_host_f64, to_host_stored, torch_mod

pytestmark = pytest.mark.gpu

DT16 = [wl.F16, wl.BF16]


def nhwc(a):
    return np.ascontiguousarray(np.transpose(a, (0, 2, 3, 1)))


def nchw(a):
    return np.ascontiguousarray(np.transpose(a, (0, 3, 1, 2)))


@pytest.mark.parametrize("dtype", [wl.F32, wl.F16, wl.BF16])
def test_convert_layout_both_directions_and_filters(dtype):
    torch = torch_mod()
    for (A, Bd, S) in [(3, 40, 169), (2, 7, 33), (5, 96, 25), (1, 1, 1), (2, 33, 64)]:
        x = wl.to_storage(wl.draw(("normal", 1.0), (A, Bd, S), 11), dtype)
        d_in = to_device(x, dtype)
        d_out = empty_out((A, S, Bd), dtype)
        B.conv_convert_layout(A, Bd, S, dtype, d_in, d_out)
        torch.cuda.synchronize()
        got = to_host_stored(d_out, dtype)
        assert np.array_equal(got, np.ascontiguousarray(np.transpose(x, (0, 2, 1)))), (A, Bd, S)
        d_back = empty_out((A, Bd, S), dtype)
        B.conv_convert_layout(A, S, Bd, dtype, d_out, d_back)
        torch.cuda.synchronize()
        assert np.array_equal(to_host_stored(d_back, dtype), x)


@pytest.mark.parametrize("dtype", [wl.F32, wl.F16, wl.BF16])
def test_maxpool_on_every_layout_pair(dtype):
    torch = torch_mod()
    for (N, C, H, W, win, stride) in [(2, 16, 27, 27, 3, 2), (3, 7, 9, 11, 2, 1), (1, 96, 55, 55, 3, 2)]:
        x = wl.to_storage(wl.draw(("normal", 1.0), (N, C, H, W), 5), dtype)
        ref = oracle.maxpool_fwd(wl.storage_to_f64(x, dtype), win=win, stride=stride)
        for in_nhwc in (False, True):
            for out_nhwc in (False, True):
                src = to_device(nhwc(x) if in_nhwc else x, dtype)
                shape = ref.shape if not out_nhwc else (ref.shape[0], ref.shape[2], ref.shape[3], ref.shape[1])
                out = empty_out(shape, dtype)
                B.maxpool_fwd_layout(N, C, H, W, win, stride, dtype, in_nhwc, out_nhwc, src, out)
                torch.cuda.synchronize()
                got = to_host_f64(out, dtype)
                if out_nhwc:
                    got = nchw(got)
                assert np.array_equal(got, ref), (N, C, H, W, in_nhwc, out_nhwc)


class NhwcCase:
    def __init__(self, shape, dtype, data, out_nhwc, relu=True):
        self.shape, self.dtype, self.out_nhwc = shape, dtype, out_nhwc
        self.desc = B.desc_of(shape, dtype, relu=relu, in_nhwc=True, out_nhwc=out_nhwc, filt_krsc=True)
        self.d_in = to_device(nhwc(data["in"]), dtype)
        self.d_filt = to_device(nhwc(data["filt"]), dtype)  # [K][C][R][S] -> [K][R][S][C]
        self.d_bias = to_device(data["bias"], wl.F32)
        self.ref = oracle.conv_fwd(wl.storage_to_f64(data["in"], dtype), wl.storage_to_f64(data["filt"], dtype),
                                   data["bias"].astype(np.float64), stride=shape.stride, pad=shape.pad, relu=relu)
        need = max(256, B.conv_workspace_bytes(self.desc))
        self.ws = torch_mod().empty(need, dtype=torch_mod().uint8, device="cuda")

    def run(self, variant=None):
        s = self.shape
        oshape = (s.N, s.OH, s.OW, s.K) if self.out_nhwc else s.out_shape()
        out = empty_out(oshape, self.dtype)
        if variant is not None:
            B.conv_force_variant(self.desc, variant)
        try:
            B.conv_fwd_ws(self.desc, self.d_in, self.d_filt, self.d_bias, out, self.ws, self.ws.numel())
            torch_mod().cuda.synchronize()
        finally:
            if variant is not None:
                B.conv_force_variant(self.desc, -1)
        got = to_host_f64(out, self.dtype)
        return nchw(got) if self.out_nhwc else got

    def names(self):
        return [B.conv_variant_name(self.desc, i) for i in range(B.conv_variant_count(self.desc))]


NHWC_SHAPES = [
    ConvShape(2, 16, 9, 11, 40, 3, 3, 1, 1),     # ragged K and pixel tiles, padding by tap mask
    ConvShape(3, 24, 13, 13, 64, 3, 3, 1, 1),    # C = 24: a 64-element step straddles window taps
    ConvShape(2, 8, 15, 15, 32, 5, 5, 1, 2),     # 5x5 window, tap mask with 25 bits
    ConvShape(1, 8, 20, 21, 24, 7, 7, 2, 3),     # 7x7 stride 2: row/column masks
    ConvShape(2, 32, 12, 12, 200, 1, 1, 1, 0),   # pointwise, no padding
    ConvShape(2, 96, 27, 27, 96, 5, 5, 1, 2),    # second layer of the stack at reduced width
    ConvShape(2, 40, 6, 6, 64, 3, 3, 2, 0),      # stride 2 without padding, 8 output pixels in all
    ConvShape(3, 64, 13, 13, 40, 3, 3, 1, 1),    # window kernel: one band per image, ragged K
    ConvShape(2, 128, 14, 10, 72, 3, 3, 1, 0),   # window kernel: no padding, K over two 64-row tiles, four chunks
    ConvShape(1, 64, 20, 20, 72, 3, 3, 1, 1),    # window kernel: bands of 9, 9 and 2 rows, K over two 64-row tiles
    ConvShape(1, 8, 1, 1, 8, 1, 1, 1, 0),        # one pixel, one channel vector: far below the smallest tile
    ConvShape(1, 16, 34, 3, 8, 3, 3, 4, 1),      # 9 output pixels, stride 4
]


@pytest.mark.parametrize("out_nhwc", [False, True])
@pytest.mark.parametrize("dtype", DT16)
@pytest.mark.parametrize("si", range(len(NHWC_SHAPES)))
def test_every_nhwc_variant(si, dtype, out_nhwc):
    shape = NHWC_SHAPES[si]
    icase = NhwcCase(shape, dtype, wl.small_int_case(shape, dtype, 900 + si), out_nhwc)
    rdata = {
        "in": wl.to_storage(wl.draw(("uniform", -1.0, 1.0), shape.in_shape(), 950 + si), dtype),
        "filt": wl.to_storage(wl.draw(("normal", wl.he_sigma(shape)), shape.filt_shape(), 951 + si), dtype),
        "bias": wl.draw(("uniform", -0.1, 0.1), (shape.K,), 952 + si),
    }
    rcase = NhwcCase(shape, dtype, rdata, out_nhwc)
    names = icase.names()
    assert names and all(n.startswith("nhwc_") for n in names), names
    exp_int = wl.storage_to_f64(wl.to_storage(icase.ref.astype(np.float32), dtype), dtype)
    for vi, name in enumerate(names):
        print("  variant %s on %s" % (name, shape), flush=True)
        got = icase.run(variant=vi)
        bad = np.argwhere(got != exp_int)
        assert bad.size == 0, "%s: %d mismatches, first at %s" % (name, len(bad), tuple(bad[0]))
        got = rcase.run(variant=vi)
        assert np.all(np.isfinite(got))
        err = oracle.max_normalised_error(got, rcase.ref)
        assert err <= TOL[dtype], "%s: error %.3g" % (name, err)


def test_layout_flags_without_a_kernel_are_refused():
    # fp32 has no channel-innermost kernel, and neither has a channel count that is no multiple of 8
    d = B.desc_of(ConvShape(1, 16, 8, 8, 16, 3, 3, 1, 1), wl.F32, in_nhwc=True, filt_krsc=True)
    assert B.conv_variant_count(d) == 0
    d = B.desc_of(ConvShape(1, 12, 8, 8, 16, 3, 3, 1, 1), wl.F16, in_nhwc=True, filt_krsc=True)
    assert B.conv_variant_count(d) == 0
    d = B.desc_of(ConvShape(1, 16, 8, 8, 16, 3, 3, 1, 1), wl.F16, in_nhwc=True)  # filters still [K][C][R][S]
    assert B.conv_variant_count(d) == 0


def _pool_rule(x, win, stride):
    """The pooling rule the library documents, written out: scan the window row by row, keep the first of equal values
    (so the sign of a zero result is that of the first zero), and let a NaN anywhere in the window be the result."""
    N, C, H, W = x.shape
    OH, OW = (H - win) // stride + 1, (W - win) // stride + 1
    out = np.empty((N, C, OH, OW), dtype=x.dtype)
    for n in range(N):
        for c in range(C):
            for oy in range(OH):
                for ox in range(OW):
                    m = x[n, c, oy * stride, ox * stride]
                    for r in range(win):
                        for s in range(win):
                            v = x[n, c, oy * stride + r, ox * stride + s]
                            if v > m or v != v:
                                m = v
                    out[n, c, oy, ox] = m
    return out


@pytest.mark.parametrize("dtype", [wl.F32, wl.F16, wl.BF16])
def test_maxpool_nan_and_signed_zero_on_every_path(dtype):
    # NaN in a tap that is not the window's first, and windows whose maximum is a zero met first as -0 or first as +0:
    # every pooling kernel (planar, channel-innermost 8 channels at a time, the two converting ones) must follow one rule
    torch = torch_mod()
    N, C, H, W = 2, 16, 9, 9
    x = -np.abs(wl.draw(("normal", 1.0), (N, C, H, W), 21)).astype(np.float32) - 0.5   # all negative: zeros are maxima
    x[0, :, 1, 1] = np.nan          # inside window (0,0) at tap (1,1); also tap (1,1)->(1,?)... of no other stride-2 window start
    x[0, :, 4, 6] = -0.0            # window (1,2) (rows 2-4, cols 4-6) and (2,2), (1,3), (2,3): -0 met first
    x[0, :, 4, 7] = 0.0
    x[1, :, 2, 2] = 0.0             # window (0,0) and (0,1), (1,0), (1,1) of image 1: +0 met first
    x[1, :, 2, 3] = -0.0
    x[1, :, 6, 5] = np.nan          # last tap of window (2,... ) rows 4-6
    stored = wl.to_storage(x, dtype)
    as_f = wl.storage_to_f64(stored, dtype)
    want = _pool_rule(as_f, 3, 2)
    assert np.isnan(want[0, 0, 0, 0]) and np.signbit(want[0, 0, 1, 2]) and not np.signbit(want[1, 0, 0, 0])
    for in_nhwc in (False, True):
        for out_nhwc in (False, True):
            src = to_device(nhwc(stored) if in_nhwc else stored, dtype)
            oshape = want.shape if not out_nhwc else (N, want.shape[2], want.shape[3], C)
            out = empty_out(oshape, dtype)
            B.maxpool_fwd_layout(N, C, H, W, 3, 2, dtype, in_nhwc, out_nhwc, src, out)
            torch.cuda.synchronize()
            got = to_host_f64(out, dtype)
            got = nchw(got) if out_nhwc else got
            assert np.array_equal(np.isnan(got), np.isnan(want)), (in_nhwc, out_nhwc)
            ok = ~np.isnan(want)
            assert np.array_equal(got[ok], want[ok]) and np.array_equal(np.signbit(got[ok]), np.signbit(want[ok])), (in_nhwc, out_nhwc)
    # a channel-innermost tensor that is not 16-byte aligned takes the element-wise kernel instead of the 16-byte one
    if dtype != wl.F32:
        base = torch.zeros(N * H * W * C + 8, dtype=torch.int16, device="cuda")
        view = base[4:4 + N * H * W * C]   # 8 bytes past a 16-byte boundary
        view.copy_(to_device(nhwc(stored), dtype).view(torch.int16).reshape(-1))
        out = empty_out((N, want.shape[2], want.shape[3], C), dtype)
        B.maxpool_fwd_layout(N, C, H, W, 3, 2, dtype, True, True, view, out)
        torch.cuda.synchronize()
        got = nchw(to_host_f64(out, dtype))
        assert np.array_equal(got, want, equal_nan=True)
