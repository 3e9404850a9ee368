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


def max_row_rel_l2(a, b):
    """max over rows i of ||a_i - b_i|| / ||b_i|| (rows = the second-to-last axis flattened out): one wrong row of
    a wide batch shows here while it would drown in the batch-wide norm."""
    import numpy as np
    a = np.asarray(a, dtype=np.float64).reshape(-1, np.shape(a)[-1])
    b = np.asarray(b, dtype=np.float64).reshape(-1, np.shape(b)[-1])
    return float(np.max(np.linalg.norm(a - b, axis=1) / np.maximum(np.linalg.norm(b, axis=1), 1e-300)))


@pytest.fixture(scope="session")
def lib():
    """The C-ABI library through its Python binding; fails loudly if it is not built."""
    from paper_2605_02189_amd import binding
    return binding
