import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def rel_err(got, ref):
    """max_i |g_i - r_i| / max(|r_i|, rms(r)): element-wise relative error with the layer's RMS
    as the floor, so that outputs that are ~0 by cancellation do not blow the ratio up."""
    import numpy as np
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    den = np.maximum(np.abs(ref), max(rms, 1e-300))
    return float(np.max(np.abs(got - ref) / den)) if ref.size else 0.0
