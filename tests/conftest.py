import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def tiny():
    import numpy as np
    import workload as wl
    from oracle.llama import as_dtype
    sh = wl.TINY
    return sh, as_dtype(wl.make_weights(sh), np.float64), wl.make_prompt(sh)
