"""Error metrics used to compare a computed tensor with the oracle's.

Outputs of linear attention are weighted means of zero-mean values: they are
small and change sign, so a purely element-wise relative error is unbounded
near zeros.  The two figures used throughout are therefore

  rel_l2  = ||g - o||_2 / ||o||_2
  max_rel = max_i |g_i - o_i| / max(|o_i|, rms(o)),   rms(o) = ||o||_2 / sqrt(n)

both taken per tensor in float64.
"""
from __future__ import annotations

import numpy as np


def rel_l2(got, ref) -> float:
    g = np.asarray(got, dtype=np.float64).ravel()
    o = np.asarray(ref, dtype=np.float64).ravel()
    den = np.linalg.norm(o)
    num = np.linalg.norm(g - o)
    if den == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return float(num / den)


def max_rel(got, ref) -> float:
    g = np.asarray(got, dtype=np.float64).ravel()
    o = np.asarray(ref, dtype=np.float64).ravel()
    if o.size == 0:
        return 0.0
    rms = np.linalg.norm(o) / np.sqrt(o.size)
    diff = np.abs(g - o)
    if rms == 0.0:
        return 0.0 if not diff.any() else float("inf")
    return float(np.max(diff / np.maximum(np.abs(o), rms)))


# Tolerances: bf16 tokens with fp32 accumulation, and the fp32 validation mode.
TOL = {
    "bf16": {"max_rel": 2e-2, "rel_l2": 5e-3},
    "f32": {"max_rel": 1e-5, "rel_l2": 1e-5},
}


def check(got, ref, dtype: str, what: str = "") -> dict:
    """Raise AssertionError unless both metrics are within TOL[dtype]."""
    m = {"max_rel": max_rel(got, ref), "rel_l2": rel_l2(got, ref)}
    tol = TOL[dtype]
    if not (np.isfinite(np.asarray(got, dtype=np.float64)).all()):
        raise AssertionError(f"{what}: non-finite values in result")
    if m["max_rel"] > tol["max_rel"] or m["rel_l2"] > tol["rel_l2"]:
        raise AssertionError(f"{what}: {m} exceeds {tol}")
    return m
