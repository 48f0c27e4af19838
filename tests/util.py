"""Comparison helpers shared by the tests (no arithmetic of the method itself)."""
import numpy as np

# Tolerances of the parity bar: max |y_gpu - y_oracle| / max |y_oracle| over one output tensor.
TOL = {"f32": 1e-5, "bf16": 2e-2}


def max_rel_err(got, want) -> float:
    """Normwise-max relative error: max_i |got_i - want_i| / max_i |want_i|."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    if want.size == 0:
        return 0.0
    denom = np.max(np.abs(want))
    num = np.max(np.abs(got - want))
    if denom == 0.0:
        return 0.0 if num == 0.0 else np.inf
    return float(num / denom)
