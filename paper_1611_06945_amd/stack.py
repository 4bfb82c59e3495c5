"""A fixed sequence of convolution layers with max-pools in between, run through the C ABI.

The paper's execution model for a compute graph (Section 3, "Code Generation,
Scheduling, and Execution"): every ND-Array is allocated up front, the operations
are issued in a topological order on one stream, and the outputs stay on the GPU.
Here the graph is a straight line, so the order is the list order.  PyTorch only
provides the device buffers; every operation is a call into libconvfwd.so.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

from . import binding as B
from .workloads import ConvShape


class ConvStack:
    def __init__(self, shapes: Sequence[ConvShape], dtype: int, pool_after: Sequence[int] = (), relu: bool = True,
                 pool_win: int = 3, pool_stride: int = 2):
        """`pool_after` holds 1-based layer numbers that are followed by a max-pool."""
        import torch

        self.torch = torch
        self.shapes = list(shapes)
        self.dtype = dtype
        self.pool_after = set(pool_after)
        self.pool_win, self.pool_stride = pool_win, pool_stride
        self.descs = [B.desc_of(s, dtype, relu=relu) for s in self.shapes]
        tdt = {B.CONV_F32: torch.float32, B.CONV_F16: torch.float16, B.CONV_BF16: torch.bfloat16}[dtype]
        self.conv_out: List = []
        self.pool_out: List[Optional[object]] = []
        ws_bytes = 256
        for i, (s, d) in enumerate(zip(self.shapes, self.descs)):
            self.conv_out.append(torch.empty(s.out_shape(), dtype=tdt, device="cuda"))
            if (i + 1) in self.pool_after:
                oh = (s.OH - pool_win) // pool_stride + 1
                ow = (s.OW - pool_win) // pool_stride + 1
                self.pool_out.append(torch.empty((s.N, s.K, oh, ow), dtype=tdt, device="cuda"))
            else:
                self.pool_out.append(None)
            ws_bytes = max(ws_bytes, B.conv_workspace_bytes(d))
            nxt = self.layer_output(i)
            if i + 1 < len(self.shapes):
                want = self.shapes[i + 1].in_shape()
                if tuple(nxt.shape) != tuple(want):
                    raise ValueError("layer %d produces %s but layer %d expects %s" % (i + 1, tuple(nxt.shape), i + 2, want))
        self.workspace = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")

    def layer_output(self, i: int):
        """What layer i (0-based) hands to the next one: its pooled output if a pool follows, else its own."""
        return self.pool_out[i] if self.pool_out[i] is not None else self.conv_out[i]

    def autotune(self, x, filts, biases, stream=None) -> None:
        cur = x
        for i, d in enumerate(self.descs):
            B.conv_autotune(d, cur, filts[i], biases[i], self.conv_out[i], self.workspace, self.workspace.numel(), stream)
            self._pool(i, stream)
            cur = self.layer_output(i)

    def _pool(self, i: int, stream) -> None:
        if self.pool_out[i] is not None:
            s = self.shapes[i]
            B.maxpool_fwd(s.N, s.K, s.OH, s.OW, self.pool_win, self.pool_stride, self.dtype, self.conv_out[i],
                          self.pool_out[i], stream)

    def run(self, x, filts, biases, stream=None):
        """Enqueue every layer; returns the last layer's output tensor (not synchronised)."""
        cur = x
        for i, d in enumerate(self.descs):
            B.conv_fwd_ws(d, cur, filts[i], biases[i], self.conv_out[i], self.workspace, self.workspace.numel(), stream)
            self._pool(i, stream)
            cur = self.layer_output(i)
        return cur
