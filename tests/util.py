"""Shared helpers for the tests (comparison metrics and launch facts only; no attention arithmetic)."""
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


# Workgroups of one XCD that run at the same time, by (head dimension, query rows per workgroup tile): 32 CUs times
# the workgroups a CU holds (three at d = 64: 32 KiB LDS and at most 168 registers each; two at d = 128; one with
# 256-row tiles, which take 128 KiB LDS and 512 registers per wavefront; with 64-row tiles -- the two halves of the
# K/V scan at once, twice the LDS of a 128-row tile -- two at d = 64 and one at d = 128).  Listed here by hand: the
# schedule oracle takes it as an input and the library's own figure is compared with it.
RESIDENT_PER_XCD = {(64, 128): 96, (128, 128): 64, (128, 256): 32, (64, 64): 64, (128, 64): 32}


def oracle_inputs(info, d, variant_kw=None):
    """Inputs of oracle.schedule_oracle for a launch of the library: the tile height and the kind of launch the
    library reports (its choices are pinned case by case in test_host_logic.py), the hand-listed resident count, and
    the variant's work decode."""
    kw = dict(variant_kw or {})
    out = {k: v for k, v in kw.items() if k in ("launch", "decode", "tiles_per_workgroup")}
    if kw.get("launch", "auto") == "auto":      # left open: what the library reports (persistent if it says nothing)
        out["launch"] = ("persistent", "grid")[info.get("launch", 0)]
    if out["launch"] == "grid" and "tiles_per_workgroup" not in out and "tiles_per_workgroup" in info:
        out["tiles_per_workgroup"] = info["tiles_per_workgroup"]
    out["tile_q"] = info["tile_q"]
    out["resident"] = kw.get("slots_per_domain") or RESIDENT_PER_XCD[(d, info["tile_q"])]
    return out
