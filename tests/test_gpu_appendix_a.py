"""GPU parity over the paper's whole benchmark set (Appendix A, 43 operations) at the paper's batch size of 5:
every output element against the CPU oracle, in the launch configuration the sweep bench times (autotuned
selection with workspace) and with the heuristic selection without workspace."""
import pytest

from paper_1611_06945_amd import binding as B
from paper_1611_06945_amd import workloads as wl

from gpu_util import TOL, DeviceCase, empty_out

pytestmark = pytest.mark.gpu

ROWS = list(range(43))


@pytest.mark.parametrize("dtype", [wl.F32, wl.F16, wl.BF16])
@pytest.mark.parametrize("row", ROWS)
def test_appendix_a_operation(row, dtype):
    w = wl.appendix_a(5, dtype)[row]
    case = DeviceCase(w.shape, w.dtype, w.generate(), relu=True, use_bias=True)
    print("  %s: heuristic %s / %s" % (w.name, B.conv_variant_name(case.desc, -1), B.conv_variant_name(case.desc, -2)),
          flush=True)
    e_nows = case.error(case.run(with_ws=False))
    ws = case.workspace()
    out = empty_out(w.shape.out_shape(), w.dtype)
    B.conv_autotune(case.desc, case.d_in, case.d_filt, case.d_bias, out, ws, ws.numel())
    print("  %s: autotuned %s" % (w.name, B.conv_variant_name(case.desc, -1)), flush=True)
    e_tuned = case.error(case.run(with_ws=True))
    assert e_nows <= TOL[dtype] and e_tuned <= TOL[dtype], (w.name, e_nows, e_tuned)
