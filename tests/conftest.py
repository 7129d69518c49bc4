import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_sessionfinish(session, exitstatus):
    """Leave the error measures of the floating-point parity tests next to the run's other output."""
    from tests import parity
    if not parity.measured:
        return
    out_dir = os.path.join(ROOT, "gpurun_out")
    try:
        os.makedirs(out_dir, exist_ok=True)
        with open(os.path.join(out_dir, "parity_measured.txt"), "w") as f:
            f.write("# what | rows | row measure | elementwise measure (floor %g)\n" % parity.FLOOR)
            for what, rows, er, ee in parity.measured:
                f.write("%s | %d | %.4g | %.4g\n" % (what, rows, er, ee))
    except OSError:
        pass
