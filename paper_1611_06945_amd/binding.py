"""Thin ctypes binding over libconvfwd.so: same names as include/convfwd.h, argument marshalling only.

Tensor arguments may be torch tensors (their ``data_ptr()`` is passed) or plain
integer device addresses.  ``stream`` may be None (torch's current stream if
torch is importable and a GPU is present, else the default stream), a
``torch.cuda.Stream`` or a raw ``hipStream_t`` value.

There is no fallback: if the shared library is missing the import of any
function here raises, and nothing in this module computes a convolution itself.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

_PKG = os.path.dirname(os.path.abspath(__file__))
# CONVFWD_LIB names another build of the library to load instead (the sanitizer job of the test suite)
LIB_PATH = os.environ.get("CONVFWD_LIB") or os.path.join(_PKG, "libconvfwd.so")

CONV_F32, CONV_F16, CONV_BF16 = 0, 1, 2
CONV_FLAG_RELU, CONV_FLAG_IN_NHWC, CONV_FLAG_OUT_NHWC, CONV_FLAG_FILT_KRSC, CONV_FLAG_FILT_WINOGRAD = 1, 2, 4, 8, 16
CONV_FLAG_MAXPOOL_3X3S2 = 32
CONV_FLAG_FILT_PACKED = 64
CONV_STATIC_SCRATCH_BYTES = 32 << 20
CONV_OK, CONV_EINVAL, CONV_EDTYPE, CONV_EWORKSPACE, CONV_EHIP, CONV_ENOVARIANT, CONV_EIO = 0, -1, -2, -3, -4, -5, -6


class conv_desc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("N", "C", "H", "W", "K", "R", "S", "stride", "pad", "dtype")] + [
        ("flags", ctypes.c_uint32)
    ]

    def __repr__(self):
        return "conv_desc(N=%d,C=%d,H=%d,W=%d,K=%d,R=%d,S=%d,stride=%d,pad=%d,dtype=%d,flags=%d)" % (
            self.N, self.C, self.H, self.W, self.K, self.R, self.S, self.stride, self.pad, self.dtype, self.flags)


CONV_OP_CONV, CONV_OP_MAXPOOL, CONV_OP_CONVERT = 0, 1, 2


class conv_op(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("desc", conv_desc), ("inp", ctypes.c_void_p), ("filt", ctypes.c_void_p),
                ("bias", ctypes.c_void_p), ("out", ctypes.c_void_p), ("workspace", ctypes.c_void_p),
                ("workspace_bytes", ctypes.c_size_t), ("p", ctypes.c_int32 * 9)]


class ConvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (where, strerror(status), status))


_lib = None


def lib() -> ctypes.CDLL:
    """Load libconvfwd.so (raises OSError with a build hint if it is not there)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise OSError("%s not found: build it with `python -m paper_1611_06945_amd.build`" % LIB_PATH)
        # The library and PyTorch must share ONE HIP runtime in the process (the tensors it is handed live in PyTorch's
        # context).  PyTorch ships its own copy of the runtime; loading it first makes the dynamic loader resolve the
        # library's dependency to that copy.  Loaded the other way round, two runtimes end up in the process and the
        # second one finds no device.
        import torch  # noqa: F401

        L = ctypes.CDLL(LIB_PATH)
        dp = ctypes.POINTER(conv_desc)
        vp, i32p = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32)
        L.conv_out_shape.argtypes = [dp, i32p, i32p]
        L.conv_out_shape.restype = ctypes.c_int
        L.conv_flops.argtypes = [dp]
        L.conv_flops.restype = ctypes.c_double
        L.conv_workspace_bytes.argtypes = [dp]
        L.conv_workspace_bytes.restype = ctypes.c_size_t
        L.conv_fwd.argtypes = [dp, vp, vp, vp, vp, vp]
        L.conv_fwd.restype = ctypes.c_int
        L.conv_fwd_ws.argtypes = [dp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.conv_fwd_ws.restype = ctypes.c_int
        L.conv_fwd_static.argtypes = [dp, vp, vp, vp, vp, vp]
        L.conv_fwd_static.restype = ctypes.c_int
        L.conv_autotune.argtypes = [dp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.conv_autotune.restype = ctypes.c_int
        L.conv_compare_outputs.argtypes = [ctypes.c_int32, vp, vp, ctypes.c_size_t, vp, ctypes.POINTER(ctypes.c_double)]
        L.conv_compare_outputs.restype = ctypes.c_int
        L.conv_run_ops.argtypes = [ctypes.POINTER(conv_op), ctypes.c_int32, vp, i32p]
        L.conv_run_ops.restype = ctypes.c_int
        L.conv_variant_count.argtypes = [dp]
        L.conv_variant_count.restype = ctypes.c_int
        L.conv_variant_name.argtypes = [dp, ctypes.c_int, ctypes.c_char_p, ctypes.c_size_t]
        L.conv_variant_name.restype = ctypes.c_int
        L.conv_variant_workspace.argtypes = [dp, ctypes.c_int]
        L.conv_variant_workspace.restype = ctypes.c_longlong
        L.conv_force_variant.argtypes = [dp, ctypes.c_int]
        L.conv_force_variant.restype = ctypes.c_int
        L.conv_variant_time_us.argtypes = [dp, ctypes.c_int]
        L.conv_variant_time_us.restype = ctypes.c_double
        L.conv_time_us.argtypes = [dp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp, ctypes.c_int, ctypes.POINTER(ctypes.c_double)]
        L.conv_time_us.restype = ctypes.c_int
        L.conv_cache_load.argtypes = [ctypes.c_char_p]
        L.conv_cache_load.restype = ctypes.c_int
        L.conv_cache_save.argtypes = [ctypes.c_char_p]
        L.conv_cache_save.restype = ctypes.c_int
        L.conv_cache_clear.argtypes = []
        L.conv_cache_clear.restype = None
        L.conv_coop_load_plan.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_int),
                                          ctypes.POINTER(ctypes.c_int)]
        L.conv_coop_load_plan.restype = ctypes.c_int
        L.maxpool_fwd.argtypes = [ctypes.c_int32] * 7 + [vp, vp, vp]
        L.maxpool_fwd.restype = ctypes.c_int
        L.maxpool_fwd_layout.argtypes = [ctypes.c_int32] * 9 + [vp, vp, vp]
        L.maxpool_fwd_layout.restype = ctypes.c_int
        L.conv_convert_layout.argtypes = [ctypes.c_int32] * 4 + [vp, vp, vp]
        L.conv_convert_layout.restype = ctypes.c_int
        L.conv_probe_mfma_peak.argtypes = [ctypes.c_int32, ctypes.c_int32, vp, vp, ctypes.POINTER(ctypes.c_double)]
        L.conv_probe_mfma_peak.restype = ctypes.c_int
        L.conv_probe_mfma_mix.argtypes = [ctypes.c_int32] * 5 + [vp, vp, ctypes.POINTER(ctypes.c_double),
                                          ctypes.POINTER(ctypes.c_double)]
        L.conv_probe_mfma_mix.restype = ctypes.c_int
        L.conv_probe_stream_bandwidth.argtypes = [vp, vp, ctypes.c_size_t, vp, ctypes.POINTER(ctypes.c_double)]
        L.conv_probe_stream_bandwidth.restype = ctypes.c_int
        L.conv_transformed_filter_bytes.argtypes = [dp]
        L.conv_transformed_filter_bytes.restype = ctypes.c_size_t
        L.conv_transform_filters.argtypes = [dp, vp, vp, vp]
        L.conv_transform_filters.restype = ctypes.c_int
        L.conv_strerror.argtypes = [ctypes.c_int]
        L.conv_strerror.restype = ctypes.c_char_p
        _lib = L
    return _lib


def make_desc(N, C, H, W, K, R, S, stride=1, pad=0, dtype=CONV_F32, relu=False, flags=None) -> conv_desc:
    f = (CONV_FLAG_RELU if relu else 0) if flags is None else flags
    return conv_desc(N, C, H, W, K, R, S, stride, pad, dtype, f)


def desc_of(shape, dtype=CONV_F32, relu=True, in_nhwc=False, out_nhwc=False, filt_krsc=False, filt_winograd=False,
            maxpool=False, filt_packed=False) -> conv_desc:
    """conv_desc from a workloads.ConvShape (optionally with channel-innermost tensor formats)."""
    flags = ((CONV_FLAG_RELU if relu else 0) | (CONV_FLAG_IN_NHWC if in_nhwc else 0) |
             (CONV_FLAG_OUT_NHWC if out_nhwc else 0) | (CONV_FLAG_FILT_KRSC if filt_krsc else 0) |
             (CONV_FLAG_FILT_WINOGRAD if filt_winograd else 0) | (CONV_FLAG_MAXPOOL_3X3S2 if maxpool else 0) | (CONV_FLAG_FILT_PACKED if filt_packed else 0))
    return make_desc(shape.N, shape.C, shape.H, shape.W, shape.K, shape.R, shape.S, shape.stride, shape.pad, dtype,
                     flags=flags)


def _ptr(x) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return int(x.data_ptr())
    raise TypeError("expected a torch tensor, an int device address or None, got %r" % type(x))


def _stream(stream) -> Optional[int]:
    if stream is None:
        try:
            import torch

            if torch.cuda.is_available():
                return int(torch.cuda.current_stream().cuda_stream) or None
        except ImportError:
            pass
        return None
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None


def _check(rc: int, where: str) -> int:
    if rc < 0:
        raise ConvError(rc, where)
    return rc


def strerror(status: int) -> str:
    return lib().conv_strerror(int(status)).decode()


def conv_out_shape(desc: conv_desc) -> Tuple[int, int]:
    oh, ow = ctypes.c_int32(), ctypes.c_int32()
    _check(lib().conv_out_shape(ctypes.byref(desc), ctypes.byref(oh), ctypes.byref(ow)), "conv_out_shape")
    return oh.value, ow.value


def conv_flops(desc: conv_desc) -> float:
    return float(lib().conv_flops(ctypes.byref(desc)))


def conv_workspace_bytes(desc: conv_desc) -> int:
    return int(lib().conv_workspace_bytes(ctypes.byref(desc)))


def conv_fwd(desc, inp, filt, bias, out, stream=None) -> None:
    _check(lib().conv_fwd(ctypes.byref(desc), _ptr(inp), _ptr(filt), _ptr(bias), _ptr(out), _stream(stream)), "conv_fwd")


def conv_fwd_ws(desc, inp, filt, bias, out, workspace, workspace_bytes, stream=None) -> None:
    _check(lib().conv_fwd_ws(ctypes.byref(desc), _ptr(inp), _ptr(filt), _ptr(bias), _ptr(out), _ptr(workspace),
                             int(workspace_bytes), _stream(stream)), "conv_fwd_ws")


def conv_fwd_static(desc, inp, filt, bias, out, stream=None) -> None:
    _check(lib().conv_fwd_static(ctypes.byref(desc), _ptr(inp), _ptr(filt), _ptr(bias), _ptr(out), _stream(stream)),
           "conv_fwd_static")


def conv_autotune(desc, inp, filt, bias, out, workspace=None, workspace_bytes=0, stream=None) -> None:
    _check(lib().conv_autotune(ctypes.byref(desc), _ptr(inp), _ptr(filt), _ptr(bias), _ptr(out), _ptr(workspace),
                               int(workspace_bytes), _stream(stream)), "conv_autotune")


def conv_time_us(desc, inp, filt, bias, out, workspace=None, workspace_bytes=0, stream=None, launches=100) -> float:
    us = ctypes.c_double(0.0)
    _check(lib().conv_time_us(ctypes.byref(desc), _ptr(inp), _ptr(filt), _ptr(bias), _ptr(out), _ptr(workspace),
                              int(workspace_bytes), _stream(stream), int(launches), ctypes.byref(us)), "conv_time_us")
    return float(us.value)


def conv_compare_outputs(dtype: int, got, ref, elements: int, stream=None) -> float:
    v = ctypes.c_double()
    _check(lib().conv_compare_outputs(dtype, _ptr(got), _ptr(ref), int(elements), _stream(stream), ctypes.byref(v)),
           "conv_compare_outputs")
    return v.value


def op_conv(desc, inp, filt, bias, out, workspace=None, workspace_bytes=0) -> conv_op:
    return conv_op(CONV_OP_CONV, desc, _ptr(inp), _ptr(filt), _ptr(bias), _ptr(out), _ptr(workspace), int(workspace_bytes),
                   (ctypes.c_int32 * 9)())


def op_maxpool(N, C, H, W, win, stride, dtype, in_nhwc, out_nhwc, inp, out) -> conv_op:
    return conv_op(CONV_OP_MAXPOOL, conv_desc(), _ptr(inp), None, None, _ptr(out), None, 0,
                   (ctypes.c_int32 * 9)(N, C, H, W, win, stride, dtype, int(bool(in_nhwc)), int(bool(out_nhwc))))


def op_convert(A, Bdim, S, dtype, inp, out) -> conv_op:
    return conv_op(CONV_OP_CONVERT, conv_desc(), _ptr(inp), None, None, _ptr(out), None, 0,
                   (ctypes.c_int32 * 9)(A, Bdim, S, dtype))


def conv_run_ops(ops, stream=None) -> None:
    """Enqueue a list (or a prepared ctypes array) of conv_op in order with one call into the library."""
    arr = ops if isinstance(ops, ctypes.Array) else (conv_op * len(ops))(*ops)
    failed = ctypes.c_int32(-1)
    rc = lib().conv_run_ops(arr, len(arr), _stream(stream), ctypes.byref(failed))
    if rc < 0:
        raise ConvError(rc, "conv_run_ops (operation %d)" % failed.value)


def conv_variant_count(desc) -> int:
    return _check(lib().conv_variant_count(ctypes.byref(desc)), "conv_variant_count")


def conv_variant_name(desc, idx: int) -> str:
    buf = ctypes.create_string_buffer(192)
    _check(lib().conv_variant_name(ctypes.byref(desc), int(idx), buf, len(buf)), "conv_variant_name")
    return buf.value.decode()


def conv_variant_workspace(desc, idx: int) -> int:
    return _check(int(lib().conv_variant_workspace(ctypes.byref(desc), int(idx))), "conv_variant_workspace")


def conv_force_variant(desc, idx: int) -> None:
    _check(lib().conv_force_variant(ctypes.byref(desc), int(idx)), "conv_force_variant")


def conv_variant_time_us(desc, idx: int) -> float:
    return float(lib().conv_variant_time_us(ctypes.byref(desc), int(idx)))


def conv_cache_load(path: str) -> None:
    _check(lib().conv_cache_load(os.fsencode(path)), "conv_cache_load")


def conv_cache_save(path: str) -> None:
    _check(lib().conv_cache_save(os.fsencode(path)), "conv_cache_save")


def conv_cache_clear() -> None:
    lib().conv_cache_clear()


def conv_coop_load_plan(threads: int, words: int) -> Tuple[int, bool]:
    n, g = ctypes.c_int(), ctypes.c_int()
    _check(lib().conv_coop_load_plan(int(threads), int(words), ctypes.byref(n), ctypes.byref(g)), "conv_coop_load_plan")
    return n.value, bool(g.value)


def maxpool_fwd(N, C, H, W, win, stride, dtype, inp, out, stream=None) -> None:
    _check(lib().maxpool_fwd(N, C, H, W, win, stride, dtype, _ptr(inp), _ptr(out), _stream(stream)), "maxpool_fwd")


def maxpool_fwd_layout(N, C, H, W, win, stride, dtype, in_nhwc, out_nhwc, inp, out, stream=None) -> None:
    _check(lib().maxpool_fwd_layout(N, C, H, W, win, stride, dtype, int(bool(in_nhwc)), int(bool(out_nhwc)), _ptr(inp),
                                    _ptr(out), _stream(stream)), "maxpool_fwd_layout")


def conv_convert_layout(A, Bdim, S, dtype, inp, out, stream=None) -> None:
    """out[a][s][b] = in[a][b][s]: (N,C,H*W) NCHW->NHWC, (N,H*W,C) NHWC->NCHW, (K,C,R*S) KCRS->KRSC."""
    _check(lib().conv_convert_layout(A, Bdim, S, dtype, _ptr(inp), _ptr(out), _stream(stream)), "conv_convert_layout")


def conv_transformed_filter_bytes(desc) -> int:
    return int(lib().conv_transformed_filter_bytes(ctypes.byref(desc)))


def conv_transform_filters(desc, filt, out, stream=None) -> None:
    """KCRS filters -> the ahead-of-time format whose bit `desc` carries (Winograd domain, or MFMA operand order)."""
    _check(lib().conv_transform_filters(ctypes.byref(desc), _ptr(filt), _ptr(out), _stream(stream)), "conv_transform_filters")


def conv_probe_mfma_peak(dtype: int, block: int, scratch, stream=None) -> float:
    v = ctypes.c_double()
    _check(lib().conv_probe_mfma_peak(dtype, block, _ptr(scratch), _stream(stream), ctypes.byref(v)), "conv_probe_mfma_peak")
    return v.value


def conv_probe_mfma_mix(dtype: int, block: int, waves_per_simd: int, valu_per_mfma: int, scratch, stream=None,
                        distinct_operands: bool = False):
    """(TFLOP/s, nanoseconds per MFMA and SIMD) of the issue loop at a fixed occupancy with interleaved vector-ALU work."""
    t, ns = ctypes.c_double(), ctypes.c_double()
    _check(lib().conv_probe_mfma_mix(dtype, block, waves_per_simd, valu_per_mfma, int(bool(distinct_operands)), _ptr(scratch), _stream(stream),
                                     ctypes.byref(t), ctypes.byref(ns)), "conv_probe_mfma_mix")
    return t.value, ns.value


def conv_probe_stream_bandwidth(src, dst, nbytes: int, stream=None) -> float:
    v = ctypes.c_double()
    _check(lib().conv_probe_stream_bandwidth(_ptr(src), _ptr(dst), int(nbytes), _stream(stream), ctypes.byref(v)),
           "conv_probe_stream_bandwidth")
    return v.value
