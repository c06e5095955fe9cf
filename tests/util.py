"""Shared helpers for the GPU parity tests (comparison metrics only; no attention arithmetic)."""
import numpy as np

MAX_ABS_TOL = 2e-3     # stated tolerance of the benchmark definition, fp16/bf16 inputs
REL_L2_TOL = 1e-3


def errors(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    assert np.all(np.isfinite(got)), "non-finite values in the GPU output"
    diff = got - want
    max_abs = float(np.abs(diff).max()) if diff.size else 0.0
    denom = float(np.sqrt((want * want).sum()))
    rel_l2 = float(np.sqrt((diff * diff).sum()) / denom) if denom > 0 else 0.0
    return max_abs, rel_l2


def assert_close(got, want, what=""):
    max_abs, rel_l2 = errors(got, want)
    assert max_abs <= MAX_ABS_TOL and rel_l2 <= REL_L2_TOL, (
        f"{what}: max-abs {max_abs:.3e} (tol {MAX_ABS_TOL}), rel-L2 {rel_l2:.3e} (tol {REL_L2_TOL})")
    return max_abs, rel_l2
