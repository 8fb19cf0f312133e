import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def rng():
    import numpy as np
    return np.random.default_rng(1234)


def pytest_terminal_summary(terminalreporter):
    """How the GPU's top-p sets compared with the oracle's over this run (tests/test_gpu_parity.py: check_topp)."""
    mod = sys.modules.get("tests.test_gpu_parity") or sys.modules.get("test_gpu_parity")
    st = getattr(mod, "TOPP_STATS", None)
    if st and st["heads"]:
        terminalreporter.write_line("top-p sets compared: %(heads)d heads; equal to the oracle's %(equal)d, differing only within 1e-6 "
                                    "of the threshold weight %(weight_band)d, inside the 1e-6 band on the cumulative mass %(mass_band)d" % st)
        for line in st["where"][:20]:
            terminalreporter.write_line("  not equal: " + line)
