"""Helpers of the GPU parity tests: move stored-type numpy arrays to the device and back, run the library
through its C ABI (via the ctypes binding), and compare with the CPU oracle."""
import numpy as np

import oracle
from paper_1611_06945_amd import binding as B
from paper_1611_06945_amd import workloads as wl

TOL = {wl.F32: 1e-5, wl.F16: 5e-3, wl.BF16: 5e-3}  # max normalised error allowed per storage type


def torch_mod():
    import torch

    return torch


def to_device(arr, dtype):
    torch = torch_mod()
    if dtype == wl.BF16:
        return torch.from_numpy(np.ascontiguousarray(arr).view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(arr)).cuda()


def empty_out(shape, dtype):
    torch = torch_mod()
    tdt = {wl.F32: torch.float32, wl.F16: torch.float16, wl.BF16: torch.bfloat16}[dtype]
    # poison so that an element the kernel fails to write cannot pass by accident
    return torch.full(tuple(shape), float("nan"), dtype=tdt, device="cuda")


def to_host_stored(t, dtype):
    """Device tensor -> numpy array in the storage representation of workloads.to_storage."""
    torch = torch_mod()
    if dtype == wl.BF16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def to_host_f64(t, dtype):
    return wl.storage_to_f64(to_host_stored(t, dtype), dtype)


class DeviceCase:
    """One convolution problem resident on the GPU, with its oracle result computed lazily on the CPU."""

    def __init__(self, shape, dtype, data, relu=True, use_bias=True):
        self.shape, self.dtype, self.relu, self.use_bias = shape, dtype, relu, use_bias
        self.data = data
        self.desc = B.desc_of(shape, dtype, relu=relu)
        self.d_in = to_device(data["in"], dtype)
        self.d_filt = to_device(data["filt"], dtype)
        self.d_bias = to_device(data["bias"], wl.F32) if use_bias else None
        self._ref = None
        self._ws = None

    def ref(self):
        if self._ref is None:
            self._ref = oracle.conv_fwd(
                wl.storage_to_f64(self.data["in"], self.dtype), wl.storage_to_f64(self.data["filt"], self.dtype),
                self.data["bias"].astype(np.float64) if self.use_bias else None,
                stride=self.shape.stride, pad=self.shape.pad, relu=self.relu)
        return self._ref

    def workspace(self):
        torch = torch_mod()
        need = B.conv_workspace_bytes(self.desc)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
        return self._ws

    def run(self, variant=None, with_ws=True):
        """Run through the C ABI; returns the device output tensor (synchronised)."""
        torch = torch_mod()
        out = empty_out(self.shape.out_shape(), self.dtype)
        if variant is not None:
            B.conv_force_variant(self.desc, variant)
        try:
            if with_ws:
                ws = self.workspace()
                B.conv_fwd_ws(self.desc, self.d_in, self.d_filt, self.d_bias, out, ws, ws.numel())
            else:
                B.conv_fwd(self.desc, self.d_in, self.d_filt, self.d_bias, out)
            torch.cuda.synchronize()
        finally:
            if variant is not None:
                B.conv_force_variant(self.desc, -1)
        return out

    def error(self, out):
        got = to_host_f64(out, self.dtype)
        assert np.all(np.isfinite(got)), "output holds NaN/Inf (unwritten or overflowed elements)"
        return oracle.max_normalised_error(got, self.ref())

    def variant_names(self):
        return [B.conv_variant_name(self.desc, i) for i in range(B.conv_variant_count(self.desc))]
