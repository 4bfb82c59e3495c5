"""GPU parity of the packed-filter window kernels (fp16/bf16): the explicit filter conversion into MFMA operand order
and every kernel that reads it, element by element against the CPU oracle through the C ABI.

The oracle only knows the paper's layouts; host-side numpy transposes carry the data to the formats the descriptor
names.  The expected packed tensor is rebuilt here from the documented order ([32-row block][16-channel group][tap]
[half][row][8 channels]) with plain numpy indexing.
"""
import sys

import numpy as np
import pytest

import oracle
from paper_1611_06945_amd import binding as B
from paper_1611_06945_amd import workloads as wl
from paper_1611_06945_amd.workloads import ConvShape

from gpu_util import TOL, empty_out, to_device, to_host_f64, to_host_stored, torch_mod

pytestmark = pytest.mark.gpu

DT16 = [wl.F16, wl.BF16]


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def nhwc(a):
    return np.ascontiguousarray(np.transpose(a, (0, 2, 3, 1)))


def nchw(a):
    return np.ascontiguousarray(np.transpose(a, (0, 3, 1, 2)))


def pack_on_host(filt):
    """[K][C][R][S] stored elements -> [ceil(K/32)][C/16][R*S][2][32][8], zero rows past K."""
    K, C, R, S = filt.shape
    KB = (K + 31) // 32
    f = np.zeros((KB * 32, C, R * S), dtype=filt.dtype)
    f[:K] = filt.reshape(K, C, R * S)
    f = f.reshape(KB, 32, C // 16, 2, 8, R * S)          # rb, m, c16, g, j, t
    return np.ascontiguousarray(np.transpose(f, (0, 2, 5, 3, 1, 4)))  # rb, c16, t, g, m, j


class PackedCase:
    def __init__(self, shape, dtype, data, out_nhwc, relu=True, use_bias=True):
        torch = torch_mod()
        self.shape, self.dtype, self.out_nhwc = shape, dtype, out_nhwc
        self.desc = B.desc_of(shape, dtype, relu=relu, in_nhwc=True, out_nhwc=out_nhwc, filt_packed=True)
        self.d_in = to_device(nhwc(data["in"]), dtype)
        d_kcrs = to_device(data["filt"], dtype)
        nbytes = B.conv_transformed_filter_bytes(self.desc)
        assert nbytes == pack_on_host(data["filt"]).nbytes, (nbytes, shape)
        self.d_filt = torch.full((nbytes // 2,), -1, dtype=torch.int16, device="cuda")
        B.conv_transform_filters(self.desc, d_kcrs, self.d_filt)
        torch.cuda.synchronize()
        self.packed_ok = np.array_equal(self.d_filt.cpu().numpy().view(np.uint16),
                                        pack_on_host(data["filt"]).view(np.uint16).ravel())
        self.d_bias = to_device(data["bias"], wl.F32) if use_bias else None
        self.ref = oracle.conv_fwd(wl.storage_to_f64(data["in"], dtype), wl.storage_to_f64(data["filt"], dtype),
                                   data["bias"].astype(np.float64) if use_bias else None, stride=shape.stride,
                                   pad=shape.pad, relu=relu)

    def run(self, variant=None):
        s = self.shape
        oshape = (s.N, s.OH, s.OW, s.K) if self.out_nhwc else s.out_shape()
        out = empty_out(oshape, self.dtype)
        if variant is not None:
            B.conv_force_variant(self.desc, variant)
        try:
            B.conv_fwd(self.desc, self.d_in, self.d_filt, self.d_bias, out)
            torch_mod().cuda.synchronize()
        finally:
            if variant is not None:
                B.conv_force_variant(self.desc, -1)
        got = to_host_f64(out, self.dtype)
        return nchw(got) if self.out_nhwc else got

    def names(self):
        return [B.conv_variant_name(self.desc, i) for i in range(B.conv_variant_count(self.desc))]


PACKED_SHAPES = [
    ConvShape(3, 64, 13, 13, 40, 3, 3, 1, 1),    # one chunk of 64 channels, K below one 64-row tile, tiles straddle images
    ConvShape(5, 128, 13, 13, 96, 3, 3, 1, 1),   # two chunks; 845 pixels: ragged last pixel tile; K = 1.5 tiles
    ConvShape(2, 128, 14, 10, 72, 3, 3, 1, 0),   # no padding: no shared border at all
    ConvShape(1, 64, 20, 20, 72, 3, 3, 1, 1),    # one image, wider rows
    ConvShape(2, 192, 7, 9, 130, 3, 3, 1, 2),    # border as wide as the window's reach (pad = R - 1), three chunks
    ConvShape(4, 32, 5, 5, 8, 3, 3, 1, 1),       # 100 pixels over 4 tiny images: a tile covers several whole images
    ConvShape(2, 64, 30, 40, 64, 3, 3, 1, 1),    # long rows: only the variants with enough slab positions are valid
    ConvShape(2, 32, 27, 27, 40, 5, 5, 1, 2),    # 5x5, the stack's second layer at reduced width
    ConvShape(3, 96, 15, 11, 64, 5, 5, 1, 1),    # 5x5, border narrower than half the window, three chunks of 32
    ConvShape(1, 64, 9, 9, 33, 5, 5, 1, 0),      # 5x5 without padding, 25 output pixels
    ConvShape(2, 48, 9, 11, 40, 3, 3, 1, 1),     # 48 channels: only the chunks of 16 divide them (no split over waves)
    ConvShape(3, 16, 12, 12, 24, 5, 5, 1, 2),    # 5x5 over a single group of 16 channels
    ConvShape(2, 96, 28, 28, 32, 3, 3, 1, 1),    # rows of 28 pixels: the 32-row tiles with 256 slab positions
]


@pytest.mark.parametrize("out_nhwc", [False, True])
@pytest.mark.parametrize("dtype", DT16)
@pytest.mark.parametrize("si", range(len(PACKED_SHAPES)))
def test_every_packed_variant(si, dtype, out_nhwc):
    shape = PACKED_SHAPES[si]
    if out_nhwc and shape.K % 8:
        pytest.skip("channel-innermost output needs K % 8 == 0")
    icase = PackedCase(shape, dtype, wl.small_int_case(shape, dtype, 1900 + si), out_nhwc)
    rdata = {
        "in": wl.to_storage(wl.draw(("uniform", -1.0, 1.0), shape.in_shape(), 1950 + si), dtype),
        "filt": wl.to_storage(wl.draw(("normal", wl.he_sigma(shape)), shape.filt_shape(), 1951 + si), dtype),
        "bias": wl.draw(("uniform", -0.1, 0.1), (shape.K,), 1952 + si),
    }
    rcase = PackedCase(shape, dtype, rdata, out_nhwc)
    assert icase.packed_ok and rcase.packed_ok, "conv_transform_filters does not write the documented order"
    names = icase.names()
    assert names and all(n.startswith("pwin_") for n in names), names
    exp_int = wl.storage_to_f64(wl.to_storage(icase.ref.astype(np.float32), dtype), dtype)
    for vi, name in enumerate(names):
        say("  variant %s on %s dtype %d out_nhwc %d" % (name, shape, dtype, out_nhwc))
        got = icase.run(variant=vi)
        bad = np.argwhere(got != exp_int)
        assert bad.size == 0, "%s: %d mismatches, first at %s got %r want %r" % (
            name, len(bad), tuple(bad[0]), got[tuple(bad[0])], exp_int[tuple(bad[0])])
        got = rcase.run(variant=vi)
        assert np.all(np.isfinite(got))
        err = oracle.max_normalised_error(got, rcase.ref)
        assert err <= TOL[dtype], "%s: error %.3g" % (name, err)


@pytest.mark.parametrize("dtype", DT16)
def test_packed_variants_without_bias_and_activation(dtype):
    shape = ConvShape(2, 64, 13, 13, 64, 3, 3, 1, 1)
    case = PackedCase(shape, dtype, wl.small_int_case(shape, dtype, 1990), True, relu=False, use_bias=False)
    exp = wl.storage_to_f64(wl.to_storage(case.ref.astype(np.float32), dtype), dtype)
    assert (exp < 0).any()
    for vi, name in enumerate(case.names()):
        say("  variant %s, no bias, identity activation" % name)
        assert np.array_equal(case.run(variant=vi), exp), name


@pytest.mark.parametrize("li", [1, 2, 3, 4])
def test_stack_layers_at_full_size_on_sampled_outputs(li):
    """Layers 2-5 of the five-layer stack (batch 20, fp16) on every packed variant: sampled outputs against the oracle."""
    w = wl.config5_layers(20, wl.F16)[li]
    shape = w.shape
    rng = np.random.default_rng(7000 + li)
    data = {
        "in": wl.to_storage(np.abs(wl.draw(("normal", 1.0), shape.in_shape(), 7100 + li)), wl.F16),
        "filt": wl.to_storage(wl.draw(("normal", wl.he_sigma(shape)), shape.filt_shape(), 7200 + li), wl.F16),
        "bias": wl.draw(("uniform", -0.1, 0.1), (shape.K,), 7300 + li),
    }
    torch = torch_mod()
    desc = B.desc_of(shape, wl.F16, relu=True, in_nhwc=True, out_nhwc=True, filt_packed=True)
    d_in = to_device(nhwc(data["in"]), wl.F16)
    d_filt = torch.empty(B.conv_transformed_filter_bytes(desc) // 2, dtype=torch.int16, device="cuda")
    B.conv_transform_filters(desc, to_device(data["filt"], wl.F16), d_filt)
    d_bias = to_device(data["bias"], wl.F32)
    n_out = shape.N * shape.K * shape.OH * shape.OW
    # the first and last pixel of the batch, and a random sample in between
    idx = np.unique(np.concatenate([np.arange(64), n_out - 1 - np.arange(64), rng.integers(0, n_out, 6000)])).astype(np.int64)
    ref = oracle.conv_fwd_points(wl.storage_to_f64(data["in"], wl.F16), wl.storage_to_f64(data["filt"], wl.F16),
                                 data["bias"].astype(np.float64), idx, stride=1, pad=shape.pad, relu=True)
    scale = max(float(np.max(np.abs(ref))), 1e-30)
    names = [B.conv_variant_name(desc, i) for i in range(B.conv_variant_count(desc))]
    assert names
    for vi, name in enumerate(names):
        say("  %s on %s" % (name, w.name))
        out = empty_out((shape.N, shape.OH, shape.OW, shape.K), wl.F16)
        B.conv_force_variant(desc, vi)
        try:
            B.conv_fwd(desc, d_in, d_filt, d_bias, out)
            torch.cuda.synchronize()
        finally:
            B.conv_force_variant(desc, -1)
        got = nchw(to_host_f64(out, wl.F16))
        assert np.all(np.isfinite(got)), name
        err = float(np.max(np.abs(got.ravel()[idx] - ref))) / scale
        assert err <= TOL[wl.F16], "%s: error %.3g" % (name, err)
