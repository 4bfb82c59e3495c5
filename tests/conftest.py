import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GOLDEN = os.path.join(ROOT, "tests", "golden")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def read_appendix_a():
    """Rows of the paper's Appendix A table as dicts (see tests/golden/appendix_a_ops.txt)."""
    rows = []
    with open(os.path.join(GOLDEN, "appendix_a_ops.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            t = line.split()
            rows.append(dict(ksz=int(t[0]), stride=int(t[1]), oc=int(t[2]), b=int(t[3]),
                             in_y=int(t[4]), in_x=int(t[5]), in_c=int(t[6]),
                             out_y=int(t[7]), out_x=int(t[8]), out_c=int(t[9]),
                             flops=float(t[10]), flops_text=t[10], pad=int(t[11])))
    return rows


@pytest.fixture(scope="session")
def appendix_a():
    return read_appendix_a()
