"""Seeded synthetic inputs and the benchmark shapes.

This module is shared by the tests, the bench and the smoke check to feed the
same bits to the GPU library and to the CPU oracle.  It holds no convolution
arithmetic: only shapes, random draws and the rounding of drawn values to the
storage type.  It imports neither the HIP binding nor the oracle.

The paper measures on pseudo-random, all-non-zero noise and takes only layer
*shapes* from AlexNet / NiN / GoogLeNet-v1 (Section 4 "Results", Experimental
Setup; Appendix A), so synthetic data stands in for nothing external here.
Draws come from numpy's PCG64 (`default_rng(seed)`) in float64, are cast to
float32, and for 16-bit storage are rounded once (nearest-even) to fp16 / bf16.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List, Optional, Tuple

import numpy as np

F32, F16, BF16 = 0, 1, 2  # storage dtype codes; the values of conv_dtype in include/convfwd.h
DTYPE_NAMES = {F32: "f32", F16: "f16", BF16: "bf16"}
DTYPE_BYTES = {F32: 4, F16: 2, BF16: 2}


@dataclass(frozen=True)
class ConvShape:
    """One convolution layer: in [N,C,H,W] * filt [K,C,R,S] -> out [N,K,OH,OW]."""

    N: int
    C: int
    H: int
    W: int
    K: int
    R: int
    S: int
    stride: int = 1
    pad: int = 0

    @property
    def OH(self) -> int:
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def OW(self) -> int:
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    @property
    def flops(self) -> int:
        """FLOP convention of Appendix A: 2 * N * K * OH * OW * C * R * S (bias and ReLU not counted)."""
        return 2 * self.N * self.K * self.OH * self.OW * self.C * self.R * self.S

    def algorithmic_bytes(self, dtype: int, bias: bool = True) -> int:
        """Every input, filter, bias and output element moved exactly once."""
        e = DTYPE_BYTES[dtype]
        n_in = self.N * self.C * self.H * self.W
        n_f = self.K * self.C * self.R * self.S
        n_out = self.N * self.K * self.OH * self.OW
        return (n_in + n_f + n_out) * e + (4 * self.K if bias else 0)

    def in_shape(self) -> Tuple[int, int, int, int]:
        return (self.N, self.C, self.H, self.W)

    def filt_shape(self) -> Tuple[int, int, int, int]:
        return (self.K, self.C, self.R, self.S)

    def out_shape(self) -> Tuple[int, int, int, int]:
        return (self.N, self.K, self.OH, self.OW)

    def with_batch(self, n: int) -> "ConvShape":
        return replace(self, N=n)


# ---------------------------------------------------------------------------
# rounding of drawn values to the storage type (input preparation only)
# ---------------------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns the 16-bit patterns as uint16."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (b >> np.uint32(16)) & np.uint32(1)
    r = (b + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(x32: np.ndarray, dtype: int) -> np.ndarray:
    """Array in the storage type: float32, float16, or uint16 holding bf16 patterns."""
    x32 = np.ascontiguousarray(x32, dtype=np.float32)
    if dtype == F32:
        return x32
    if dtype == F16:
        return x32.astype(np.float16)
    if dtype == BF16:
        return f32_to_bf16_bits(x32)
    raise ValueError("unknown dtype code %r" % (dtype,))


def storage_to_f64(stored: np.ndarray, dtype: int) -> np.ndarray:
    """Exact widening of stored values to float64 (what the oracle is fed)."""
    if dtype == BF16:
        return bf16_bits_to_f32(stored).astype(np.float64)
    return np.asarray(stored).astype(np.float64)


# ---------------------------------------------------------------------------
# distributions
# ---------------------------------------------------------------------------

def draw(dist: Tuple, shape, seed: int) -> np.ndarray:
    """dist = ("uniform", lo, hi) | ("normal", sigma) | ("halfnormal", sigma) | ("int", lo, hi) -> float32."""
    rng = np.random.default_rng(int(seed))
    kind = dist[0]
    if kind == "uniform":
        x = rng.uniform(dist[1], dist[2], size=shape)
    elif kind == "normal":
        x = rng.normal(0.0, dist[1], size=shape)
    elif kind == "halfnormal":
        x = np.abs(rng.normal(0.0, dist[1], size=shape))
    elif kind == "int":  # integers in [lo, hi], for the order-independent bit-exact cases
        x = rng.integers(dist[1], dist[2] + 1, size=shape).astype(np.float64)
    else:
        raise ValueError("unknown distribution %r" % (kind,))
    return x.astype(np.float32)


def he_sigma(shape: ConvShape) -> float:
    return float(np.sqrt(2.0 / (shape.C * shape.R * shape.S)))


@dataclass(frozen=True)
class Workload:
    """A named layer of one of the benchmark configurations."""

    name: str
    config: int  # 1..5, the position in the list of benchmark configurations
    layer: int  # 0 for single-layer configurations, 1..5 inside the stack
    shape: ConvShape
    dtype: int
    in_dist: Tuple
    filt_dist: Tuple
    bias_dist: Tuple = ("uniform", -0.1, 0.1)
    paper_row: Optional[str] = None  # Appendix A row (KSZ,S,OC,in->out) this shape is, if any

    def seeds(self) -> Tuple[int, int, int]:
        base = 1000 * self.config + 100 * self.layer
        return base, base + 1, base + 2

    def generate(self) -> Dict[str, np.ndarray]:
        """Stored-type arrays 'in', 'filt' and float32 'bias' (bias is always fp32)."""
        s_in, s_f, s_b = self.seeds()
        return {
            "in": to_storage(draw(self.in_dist, self.shape.in_shape(), s_in), self.dtype),
            "filt": to_storage(draw(self.filt_dist, self.shape.filt_shape(), s_f), self.dtype),
            "bias": draw(self.bias_dist, (self.shape.K,), s_b),
        }


_MID = ConvShape(1, 256, 13, 13, 384, 3, 3, 1, 1)
_FIRST = ConvShape(20, 3, 227, 227, 96, 11, 11, 4, 0)


def config1() -> Workload:
    return Workload("cfg1_toy3x3_f32", 1, 0, ConvShape(1, 3, 32, 32, 16, 3, 3, 1, 1), F32,
                    ("uniform", -1.0, 1.0), ("uniform", -1.0, 1.0))


def config2() -> Workload:
    return Workload("cfg2_pointwise_f32", 2, 0, ConvShape(5, 256, 28, 28, 128, 1, 1, 1, 0), F32,
                    ("halfnormal", 1.0), ("normal", float(np.sqrt(2.0 / 256))),
                    paper_row="1,1,128, 28x28x256 -> 28x28x128")


def config3() -> Workload:
    return Workload("cfg3_first11x11_f32", 3, 0, _FIRST, F32, ("uniform", -128.0, 128.0), ("normal", 0.01),
                    paper_row="11,4,96, 227x227x3 -> 55x55x96")


def config4(batch: int, dtype: int = F32) -> Workload:
    sh = _MID.with_batch(batch)
    return Workload("cfg4_mid3x3_n%d_%s" % (batch, DTYPE_NAMES[dtype]), 4, 0, sh, dtype,
                    ("halfnormal", 1.0), ("normal", he_sigma(sh)),
                    paper_row="3,1,384, 13x13x256 -> 13x13x384")


def config5_layers(batch: int = 20, dtype: int = F16) -> List[Workload]:
    """The five convolution layers of the stack; max-pool 3x3 stride 2 follows layers 1 and 2.

    Each layer's `in_dist` is only used when the layer is run on its own (bench
    per-layer lines); inside the stack the input is the previous layer's output.
    """
    shapes = [
        ConvShape(batch, 3, 227, 227, 96, 11, 11, 4, 0),
        ConvShape(batch, 96, 27, 27, 256, 5, 5, 1, 2),
        ConvShape(batch, 256, 13, 13, 384, 3, 3, 1, 1),
        ConvShape(batch, 384, 13, 13, 384, 3, 3, 1, 1),
        ConvShape(batch, 384, 13, 13, 256, 3, 3, 1, 1),
    ]
    rows = ["11,4,96, 227x227x3 -> 55x55x96", "5,1,256, 27x27x96 -> 27x27x256",
            "3,1,384, 13x13x256 -> 13x13x384", "3,1,384, 13x13x384 -> 13x13x384",
            "3,1,256, 13x13x384 -> 13x13x256"]
    out = []
    for i, sh in enumerate(shapes):
        in_dist = ("uniform", -128.0, 128.0) if i == 0 else ("halfnormal", 1.0)
        out.append(Workload("cfg5_L%d_%s" % (i + 1, DTYPE_NAMES[dtype]), 5, i + 1, sh, dtype, in_dist,
                            ("normal", he_sigma(sh)), paper_row=rows[i]))
    return out


# The paper's benchmark set (Appendix A, "Benchmark Operations List"): every convolution of three ImageNet networks,
# as (KSZ, stride, OC, in_y, in_x, in_chan, pad), sorted by FLOPs as printed there.  The table prints no padding;
# `pad` is what the printed in -> out sizes imply under floor rounding.  Batch is a parameter (the paper uses 5).
_APPENDIX_A = (
    (5, 1, 32, 28, 28, 16, 2), (5, 1, 64, 14, 14, 32, 2), (1, 1, 256, 7, 7, 832, 0), (1, 1, 112, 14, 14, 512, 0),
    (1, 1, 128, 14, 14, 512, 0), (1, 1, 64, 28, 28, 256, 0), (1, 1, 64, 56, 56, 64, 0), (1, 1, 128, 14, 14, 528, 0),
    (1, 1, 144, 14, 14, 512, 0), (1, 1, 96, 28, 28, 192, 0), (1, 1, 384, 7, 7, 832, 0), (1, 1, 160, 14, 14, 512, 0),
    (1, 1, 160, 14, 14, 528, 0), (1, 1, 4096, 1, 1, 4096, 0), (1, 1, 192, 14, 14, 480, 0), (5, 1, 128, 14, 14, 32, 2),
    (3, 1, 320, 7, 7, 160, 1), (1, 1, 384, 13, 13, 384, 0), (1, 1, 128, 28, 28, 256, 0), (1, 1, 256, 14, 14, 528, 0),
    (1, 1, 96, 54, 54, 96, 0), (3, 1, 384, 7, 7, 192, 1), (3, 1, 208, 14, 14, 96, 1), (1, 1, 1000, 6, 6, 1024, 0),
    (1, 1, 1024, 6, 6, 1024, 0), (6, 1, 4096, 6, 6, 256, 0), (3, 1, 224, 14, 14, 112, 1), (1, 1, 256, 27, 27, 256, 0),
    (3, 1, 256, 14, 14, 128, 1), (5, 1, 96, 28, 28, 32, 2), (3, 1, 288, 14, 14, 144, 1), (3, 1, 128, 28, 28, 96, 1),
    (3, 1, 320, 14, 14, 160, 1), (11, 4, 96, 224, 224, 3, 0), (11, 4, 96, 227, 227, 3, 0), (7, 2, 64, 224, 224, 3, 3),
    (3, 1, 1024, 6, 6, 384, 1), (3, 1, 256, 13, 13, 384, 1), (3, 1, 384, 13, 13, 256, 1), (3, 1, 192, 28, 28, 128, 1),
    (3, 1, 384, 13, 13, 384, 1), (3, 1, 192, 56, 56, 64, 1), (5, 1, 256, 27, 27, 96, 2),
)


def appendix_a(batch: int = 5, dtype: int = F32) -> List[Workload]:
    """All 43 operations of the paper's benchmark set at one batch size, in the table's order (by FLOPs).

    Inputs: image-like U[-128,128] for the three-channel first layers, half-normal (post-ReLU activations) elsewhere;
    He-scaled normal filters; seeds 6000 + 100*row + {0,1,2}.
    """
    out = []
    for i, (ksz, st, oc, iy, ix, ic, pad) in enumerate(_APPENDIX_A):
        sh = ConvShape(batch, ic, iy, ix, oc, ksz, ksz, st, pad)
        in_dist = ("uniform", -128.0, 128.0) if ic == 3 else ("halfnormal", 1.0)
        out.append(Workload("appA_%02d_k%ds%d_%dx%dx%d_oc%d_n%d_%s" % (i, ksz, st, iy, ix, ic, oc, batch, DTYPE_NAMES[dtype]),
                            6, i, sh, dtype, in_dist, ("normal", he_sigma(sh)),
                            paper_row="%d,%d,%d, %dx%dx%d -> %dx%dx%d" % (ksz, st, oc, iy, ix, ic, sh.OH, sh.OW, oc)))
    return out


STACK_POOL_AFTER = (1, 2)  # max-pool 3x3 stride 2 follows these layers of the stack


def small_int_case(shape: ConvShape, dtype: int, seed: int) -> Dict[str, np.ndarray]:
    """Small-integer data: every partial sum is an exactly representable integer, so any
    accumulation order, tile shape or split must reproduce the oracle bit for bit."""
    return {
        "in": to_storage(draw(("int", -3, 3), shape.in_shape(), seed), dtype),
        "filt": to_storage(draw(("int", -2, 2), shape.filt_shape(), seed + 1), dtype),
        "bias": draw(("int", -4, 4), (shape.K,), seed + 2),
    }
