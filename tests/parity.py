"""Comparison rule of the GPU join against the oracle (used by the GPU tests, smoke() and bench.py's checks).

Result sets are compared exactly after sorting by (r, h, t).  The only exclusion: triples whose oracle
distance lies within 1e-4 * delta of the threshold are removed from both sides and counted.  Reported
distances must agree to 1e-4 relative (absolute floor 1e-6 for a zero distance).
"""
from __future__ import annotations

import numpy as np

import oracle

BAND = 1e-4
DIST_RTOL = 1e-4
DIST_ATOL = 1e-6


def _keys(r, h, t, N):
    return (np.asarray(r, np.int64) * N + np.asarray(h, np.int64)) * N + np.asarray(t, np.int64)


def compare(gpu: dict, ref: dict, E, Rv, p: int, delta: float, N: int) -> dict:
    """gpu/ref: dicts with arrays h, r, t, dist.  Returns a report; raises AssertionError on a mismatch."""
    gk = _keys(gpu["r"], gpu["h"], gpu["t"], N)
    rk = _keys(ref["r"], ref["h"], ref["t"], N)
    assert np.unique(gk).size == gk.size, "GPU result holds a triple more than once"
    go, ro = np.argsort(gk), np.argsort(rk)
    gk, rk = gk[go], rk[ro]
    gd = np.asarray(gpu["dist"], np.float64)[go]
    rd = np.asarray(ref["dist"], np.float64)[ro]
    band_tol = BAND * abs(delta)
    # oracle distances of GPU triples the oracle did not list (needed to decide band membership)
    only_g = ~np.isin(gk, rk)
    only_r = ~np.isin(rk, gk)
    extra_d = np.empty(0)
    if only_g.any():
        idx = go[only_g]
        extra_d = oracle.dist_triples(E, Rv, p, np.asarray(gpu["h"])[idx], np.asarray(gpu["r"])[idx],
                                      np.asarray(gpu["t"])[idx])
    bad_extra = int(np.sum(np.abs(extra_d - delta) > band_tol))
    bad_missing = int(np.sum(np.abs(rd[only_r] - delta) > band_tol))
    in_band = int(np.sum(np.abs(rd - delta) <= band_tol)) + int(np.sum(np.abs(extra_d - delta) <= band_tol))
    assert bad_extra == 0, f"{bad_extra} GPU triples are not in the oracle set (outside the boundary band)"
    assert bad_missing == 0, f"{bad_missing} oracle triples are missing from the GPU set (outside the boundary band)"
    common_g = np.isin(gk, rk)
    common_r = np.isin(rk, gk)
    dg, dr = gd[common_g], rd[common_r]
    err = np.abs(dg - dr)
    tol = np.maximum(DIST_RTOL * np.abs(dr), DIST_ATOL)
    assert np.all(err <= tol), f"distance mismatch: max rel err {np.max(err / np.maximum(np.abs(dr), 1e-30)):.3e}"
    return {"gpu_count": int(gk.size), "oracle_count": int(rk.size), "boundary_band": in_band,
            "only_gpu_in_band": int(only_g.sum()), "only_oracle_in_band": int(only_r.sum()),
            "max_rel_dist_err": float(np.max(err / np.maximum(np.abs(dr), 1e-30))) if err.size else 0.0}
