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


# Reported, never gated: lines collected here are printed at the end of the pytest run (tests/conftest.py).
DIAG_LINES = []


def elementwise_violations(got, want, tol) -> float:
    """Fraction of elements that miss |got - want| <= tol * |want| + tol * rms(want)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    if want.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(want * want)))
    return float(np.mean(np.abs(got - want) > tol * np.abs(want) + tol * rms))


def column_block_err(got, want, block: int = 64) -> float:
    """Largest over blocks of `block` columns of max |got - want| / max |want| inside that block: a wrong
    tile whose values are small against the tensor's maximum shows up here."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    worst = 0.0
    for c0 in range(0, want.shape[-1], block):
        w = want[..., c0:c0 + block]
        d = np.max(np.abs(w))
        if d > 0:
            worst = max(worst, float(np.max(np.abs(got[..., c0:c0 + block] - w)) / d))
    return worst


def diag_report(label, got, exact, faithful=None, dtype="bf16", gate_blocks=True) -> None:
    """Record the diagnostics of one output tensor: normwise-max error against the exact fp64 definition (the
    gated number), against the rounding-faithful diagnostic oracle, the worst 64-column block (gated too unless
    gate_blocks is False), and the fraction of elements outside the elementwise check."""
    tol = TOL[dtype]
    line = f"{label:58s} exact {max_rel_err(got, exact):.2e}  per-64-col {column_block_err(got, exact):.2e}  " \
           f"elementwise-miss {elementwise_violations(got, exact, tol):.1e}"
    if faithful is not None:
        line += f"  vs rounding-faithful {max_rel_err(got, faithful):.2e}"
    DIAG_LINES.append(line)
    # gated as well (the tolerance applied to every block of 64 columns against that block's own largest value): a wrong tile of
    # small values cannot hide behind the tensor's maximum
    if gate_blocks:
        assert column_block_err(got, exact) <= tol, label
