"""ctypes wrapper around ``conv_oracle.c`` -- TEST INFRASTRUCTURE ONLY.

The arithmetic lives in the C file (fp64, the paper's definition of a
convolution layer written as nested loops; Section 2 "Background" and
Appendix A).  This module only builds the shared object with gcc, widens the
caller's arrays to float64 (exact for fp32 / fp16 / bf16 values) and hands
pointers over.  Nothing here is used by, or uses, the HIP library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv_oracle.c")
# ORACLE_CONV_LIB names another build of the same source to load instead (the sanitizer job of the test suite)
_LIB_OVERRIDE = os.environ.get("ORACLE_CONV_LIB")
_LIB = _LIB_OVERRIDE or os.path.join(_HERE, "liboracle_conv.so")
_lock = threading.Lock()
_lib = None

_c_double_p = ctypes.POINTER(ctypes.c_double)
_c_int64_p = ctypes.POINTER(ctypes.c_int64)


def build(force: bool = False) -> str:
    """Compile ``conv_oracle.c`` into ``liboracle_conv.so`` (gcc -O2 -fopenmp)."""
    if _LIB_OVERRIDE:
        return _LIB
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-o", tmp, _SRC]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build())
            i = ctypes.c_int
            lib.oracle_conv_out_shape.argtypes = [i] * 6 + [ctypes.POINTER(i), ctypes.POINTER(i)]
            lib.oracle_conv_out_shape.restype = i
            lib.oracle_conv_fwd.argtypes = [i] * 9 + [_c_double_p, _c_double_p, _c_double_p, i, _c_double_p]
            lib.oracle_conv_fwd.restype = i
            lib.oracle_conv_fwd_points.argtypes = (
                [i] * 9 + [_c_double_p, _c_double_p, _c_double_p, i, ctypes.c_long, _c_int64_p, _c_double_p]
            )
            lib.oracle_conv_fwd_points.restype = i
            lib.oracle_maxpool_fwd.argtypes = [i] * 6 + [_c_double_p, _c_double_p]
            lib.oracle_maxpool_fwd.restype = i
            lib.oracle_threads.restype = i
            lib.oracle_set_threads.argtypes = [i]
            _lib = lib
    return _lib


def _f64(a, shape=None):
    a = np.ascontiguousarray(np.asarray(a, dtype=np.float64))
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError("expected shape %s, got %s" % (tuple(shape), a.shape))
    return a


def _ptr(a):
    return a.ctypes.data_as(_c_double_p)


def threads() -> int:
    return int(_load().oracle_threads())


def set_threads(n: int) -> None:
    _load().oracle_set_threads(int(n))


def conv_out_shape(H, W, R, S, stride, pad):
    """(OH, OW) = floor((H+2*pad-R)/stride)+1, likewise for W; ValueError if the window does not fit."""
    oh, ow = ctypes.c_int(), ctypes.c_int()
    if _load().oracle_conv_out_shape(H, W, R, S, stride, pad, ctypes.byref(oh), ctypes.byref(ow)):
        raise ValueError("invalid convolution geometry")
    return oh.value, ow.value


def conv_fwd(inp, filt, bias=None, *, stride=1, pad=0, relu=False):
    """Direct convolution in fp64.  inp [N,C,H,W], filt [K,C,R,S], bias [K] or None -> float64 [N,K,OH,OW]."""
    inp = _f64(inp)
    filt = _f64(filt)
    if inp.ndim != 4 or filt.ndim != 4 or inp.shape[1] != filt.shape[1]:
        raise ValueError("expected inp [N,C,H,W] and filt [K,C,R,S] with equal C")
    N, C, H, W = inp.shape
    K, _, R, S = filt.shape
    OH, OW = conv_out_shape(H, W, R, S, stride, pad)
    b = None if bias is None else _f64(bias, (K,))
    out = np.empty((N, K, OH, OW), dtype=np.float64)
    rc = _load().oracle_conv_fwd(
        N, C, H, W, K, R, S, stride, pad, _ptr(inp), _ptr(filt), None if b is None else _ptr(b),
        1 if relu else 0, _ptr(out),
    )
    if rc:
        raise ValueError("oracle_conv_fwd rejected its arguments")
    return out


def conv_fwd_points(inp, filt, bias, flat_idx, *, stride=1, pad=0, relu=False):
    """The same definition at chosen flat indices of out[N,K,OH,OW] only."""
    inp = _f64(inp)
    filt = _f64(filt)
    N, C, H, W = inp.shape
    K, C2, R, S = filt.shape
    if C != C2:
        raise ValueError("channel mismatch")
    b = None if bias is None else _f64(bias, (K,))
    idx = np.ascontiguousarray(np.asarray(flat_idx, dtype=np.int64))
    vals = np.empty(idx.shape, dtype=np.float64)
    rc = _load().oracle_conv_fwd_points(
        N, C, H, W, K, R, S, stride, pad, _ptr(inp), _ptr(filt), None if b is None else _ptr(b),
        1 if relu else 0, idx.size, idx.ctypes.data_as(_c_int64_p), _ptr(vals),
    )
    if rc:
        raise ValueError("oracle_conv_fwd_points rejected its arguments")
    return vals


def maxpool_fwd(inp, *, win=3, stride=2):
    """Per-channel spatial max-pool, no padding, floor output size.  inp [N,C,H,W] -> float64."""
    inp = _f64(inp)
    N, C, H, W = inp.shape
    if H < win or W < win:
        raise ValueError("window larger than input")
    OH, OW = (H - win) // stride + 1, (W - win) // stride + 1
    out = np.empty((N, C, OH, OW), dtype=np.float64)
    if _load().oracle_maxpool_fwd(N, C, H, W, win, stride, _ptr(inp), _ptr(out)):
        raise ValueError("oracle_maxpool_fwd rejected its arguments")
    return out


def max_normalised_error(got, ref) -> float:
    """max_i |got_i - ref_i| / max(max_j |ref_j|, 1e-30): the comparison metric of the parity tests."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if got.shape != ref.shape:
        raise ValueError("shape mismatch %s vs %s" % (got.shape, ref.shape))
    if ref.size == 0:
        return 0.0
    scale = max(float(np.max(np.abs(ref))), 1e-30)
    return float(np.max(np.abs(got - ref))) / scale
