import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # the tests load what is built; only if nothing is built yet they build it (hipcc cross-compiles without a GPU)
    from paper_2605_02189_amd.build import ensure_built
    ensure_built()


def rel_l2(a, b):
    """||a - b|| / ||b|| in float64."""
    import numpy as np
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


@pytest.fixture(scope="session")
def lib():
    """The C-ABI library through its Python binding; fails loudly if it is not built."""
    from paper_2605_02189_amd import binding
    return binding
