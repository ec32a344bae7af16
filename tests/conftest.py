import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def rel_err(got, want, floor=None):
    """max_i |got - want| / max(|want_i|, rms(want)); the parity metric of the float paths."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    if want.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(want * want))) if floor is None else floor
    den = np.maximum(np.abs(want), rms if rms > 0 else 1.0)
    return float(np.max(np.abs(got - want) / den))


@pytest.fixture(scope="session")
def rel():
    return rel_err
