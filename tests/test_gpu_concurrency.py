"""Several host threads calling the library at once, each on its own stream with its own tensors and workspace: the
results must equal those of the same calls made one after the other (and so the oracle's, which the serial calls are
checked against elsewhere)."""
import threading

import numpy as np
import pytest

from paper_1611_06945_amd import binding as B
from paper_1611_06945_amd import workloads as wl
from paper_1611_06945_amd.workloads import ConvShape

from gpu_util import TOL, to_host_stored, torch_mod
from test_gpu_parity import random_case

pytestmark = pytest.mark.gpu

JOBS = [
    (ConvShape(4, 64, 13, 13, 96, 3, 3, 1, 1), wl.F32),    # window / Winograd kernels, workspace in use
    (ConvShape(2, 3, 67, 67, 32, 11, 11, 4, 0), wl.F16),   # first-layer gather
    (ConvShape(3, 96, 14, 14, 160, 1, 1, 1, 0), wl.F32),   # pointwise, split reduction
    (ConvShape(2, 32, 27, 27, 48, 5, 5, 1, 2), wl.BF16),   # 16-bit window kernel
    (ConvShape(5, 256, 6, 6, 100, 6, 6, 1, 0), wl.F16),    # fully connected
    (ConvShape(2, 20, 12, 12, 200, 3, 3, 1, 1), wl.F32),   # implicit GEMM with ragged tiles
]


def test_threads_on_their_own_streams_match_serial_calls():
    torch = torch_mod()
    cases = [random_case(s, dt, 8000 + i) for i, (s, dt) in enumerate(JOBS)]
    serial = []
    for c in cases:
        out = c.run()
        assert c.error(out) <= TOL[c.dtype]
        serial.append(to_host_stored(out, c.dtype).copy())
    rounds = 25
    results = [[None] * rounds for _ in cases]
    errors = []

    def work(ci):
        try:
            c = cases[ci]
            stream = torch.cuda.Stream()
            tdt = {wl.F32: torch.float32, wl.F16: torch.float16, wl.BF16: torch.bfloat16}[c.dtype]
            ws = torch.empty(max(256, B.conv_workspace_bytes(c.desc)), dtype=torch.uint8, device="cuda")
            outs = [torch.empty(c.shape.out_shape(), dtype=tdt, device="cuda") for _ in range(rounds)]
            for r in range(rounds):
                if r % 2:
                    B.conv_fwd_ws(c.desc, c.d_in, c.d_filt, c.d_bias, outs[r], ws, ws.numel(), stream.cuda_stream)
                else:
                    B.conv_fwd(c.desc, c.d_in, c.d_filt, c.d_bias, outs[r], stream.cuda_stream)
            stream.synchronize()
            for r in range(rounds):
                results[ci][r] = to_host_stored(outs[r], c.dtype)
        except Exception as e:  # surfaced in the main thread
            errors.append((ci, repr(e)))

    threads = [threading.Thread(target=work, args=(i,)) for i in range(len(cases))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    for ci, c in enumerate(cases):
        with_ws = serial[ci]
        # calls without a workspace may select another variant: compare those with a serial call of the same kind
        no_ws = to_host_stored(c.run(with_ws=False), c.dtype)
        for r in range(rounds):
            want = with_ws if r % 2 else no_ws
            assert np.array_equal(results[ci][r].view(np.uint8), want.view(np.uint8)), \
                "job %d round %d differs from the serial call" % (ci, r)
