"""CPU oracle for the TransE completion join -- TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  The product path (the HIP library and its
Python binding) never does, and this package imports nothing from it.

The arithmetic lives in ``kgc_oracle.c`` (plain C, IEEE double): the triple loop
of Definition 1 / Section 3.1 with the TransE distance of Section 4.3, plus two
modes that must return the same set (early abandon; the pivot filter of
Sections 4.4-4.5).  This file marshals numpy arrays and adds the grouping rule
of Section 4.6 as plain Python for its worked example.

Pins (see tests/test_oracle_*.py): a hand-computed 3-entity case, a lattice with
a closed-form count, scipy's cdist on small inputs, symmetry / negation /
translation / norm-ordering invariants, Lemma 1 on every emitted triple,
brute force == early abandon == pivot filter, two-pointer ranges == binary
search ranges == Lemma 2's definition, the range example and group size printed
in Section 4.6, and the triple count printed in Section 5.1.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kgc_oracle.c")
_LIB = os.path.join(_HERE, "libkgc_oracle.so")
_lib = None

MODES = {"brute": 0, "abandon": 1, "pivot": 2}
RANGE_IMPLS = {"two_pointer": 0, "binary_search": 1}


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        lp = ctypes.POINTER(ctypes.c_int64)
        lib.kgco_join.restype = ctypes.c_int64
        lib.kgco_join.argtypes = [dp, ctypes.c_int64, ctypes.c_int32, dp, ctypes.c_int32, ctypes.c_int32,
                                  ctypes.c_double, ctypes.c_int32, dp, ctypes.c_int32, ctypes.c_int64,
                                  ip, ip, ip, dp, lp]
        lib.kgco_dist_triples.restype = None
        lib.kgco_dist_triples.argtypes = [dp, ctypes.c_int32, dp, ctypes.c_int32, ip, ip, ip, ctypes.c_int64, dp]
        lib.kgco_join_ab.restype = ctypes.c_int64
        lib.kgco_join_ab.argtypes = [dp, dp, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                     ctypes.c_double, ctypes.c_int64, ip, ip, ip, dp]
        lib.kgco_topk.restype = ctypes.c_int64
        lib.kgco_topk.argtypes = [dp, ctypes.c_int64, ctypes.c_int32, dp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                  ctypes.c_int64, ip, ip, ip, dp]
        lib.kgco_top1.restype = ctypes.c_int32
        lib.kgco_top1.argtypes = [dp, ctypes.c_int64, ctypes.c_int32, dp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                  ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32),
                                  ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_double)]
        lib.kgco_compute_range.restype = None
        lib.kgco_compute_range.argtypes = [dp, ctypes.c_int64, dp, ctypes.c_int64, ctypes.c_double,
                                           ctypes.c_int32, lp, lp]
        lib.kgco_num_threads.restype = ctypes.c_int32
        lib.kgco_set_num_threads.argtypes = [ctypes.c_int32]
        _lib = lib
    return _lib


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _ptr(a: np.ndarray, ty):
    return a.ctypes.data_as(ctypes.POINTER(ty))


def num_threads() -> int:
    return int(_load().kgco_num_threads())


def set_num_threads(n: int) -> None:
    _load().kgco_set_num_threads(int(n))


def join(E, Rv, p: int, delta: float, mode: str = "brute", pivot=None, range_impl: str = "two_pointer",
         cap: Optional[int] = None) -> dict:
    """All (h, r, t) with ||E[h] + Rv[r] - E[t]||_p <= delta (Definition 1; TransE distance, Section 4.3).

    ``E`` (N x d) and ``Rv`` (R x d) are widened to float64 exactly (pass the
    values the GPU sees: float32, or bfloat16 widened to float32).  Returns a
    dict with int32 arrays ``h``, ``r``, ``t`` and float64 ``dist`` sorted by
    (r, h, t), the total ``count`` and ``evaluated`` (distances started).
    """
    lib = _load()
    E64, R64 = _f64(E), _f64(Rv)
    if E64.ndim != 2 or R64.ndim != 2 or (E64.shape[1] != R64.shape[1] and E64.size and R64.size):
        raise ValueError("E must be N x d and Rv must be R x d")
    N, d = E64.shape
    R = R64.shape[0]
    pv = None if pivot is None else _f64(pivot)
    if pv is not None and pv.shape != (d,):
        raise ValueError("pivot must have d components")
    cap = int(cap) if cap is not None else 1 << 20
    while True:
        oh = np.empty(cap, np.int32); orr = np.empty(cap, np.int32); ot = np.empty(cap, np.int32)
        od = np.empty(cap, np.float64)
        ev = ctypes.c_int64(0)
        total = lib.kgco_join(_ptr(E64, ctypes.c_double), N, d, _ptr(R64, ctypes.c_double), R, int(p),
                              float(delta), MODES[mode],
                              None if pv is None else _ptr(pv, ctypes.c_double), RANGE_IMPLS[range_impl],
                              cap, _ptr(oh, ctypes.c_int32), _ptr(orr, ctypes.c_int32),
                              _ptr(ot, ctypes.c_int32), _ptr(od, ctypes.c_double), ctypes.byref(ev))
        if total < 0:
            raise ValueError("oracle rejected its arguments (p must be 1 or 2)")
        if total <= cap:
            break
        cap = int(total)
    n = int(total)
    oh, orr, ot, od = oh[:n], orr[:n], ot[:n], od[:n]
    order = np.lexsort((ot, oh, orr))
    return {"h": oh[order], "r": orr[order], "t": ot[order], "dist": od[order], "count": n,
            "evaluated": int(ev.value)}


def join_ab(A, B, p: int, delta: float, cap: Optional[int] = None) -> dict:
    """The join on connector outputs supplied by the caller (Section 4.3): all (h, r, t) with
    ||A[r][h] - B[r][t]||_p <= delta.  ``A`` is R x N x d; ``B`` is R x N x d, or 1 x N x d (or N x d) when
    connector_2 does not depend on the relation.  Same result convention as ``join``."""
    lib = _load()
    A64, B64 = _f64(A), _f64(B)
    if B64.ndim == 2:
        B64 = B64[None]
    if A64.ndim != 3 or B64.ndim != 3 or A64.shape[1:] != B64.shape[1:] or B64.shape[0] not in (1, A64.shape[0]):
        raise ValueError("A must be R x N x d and B must be R x N x d or 1 x N x d")
    R, N, d = A64.shape
    per_rel = 1 if (B64.shape[0] == R and R > 1) else 0
    cap = int(cap) if cap is not None else 1 << 20
    while True:
        oh = np.empty(cap, np.int32); orr = np.empty(cap, np.int32); ot = np.empty(cap, np.int32)
        od = np.empty(cap, np.float64)
        total = lib.kgco_join_ab(_ptr(A64, ctypes.c_double), _ptr(B64, ctypes.c_double), N, d, R, per_rel, int(p),
                                 float(delta), cap, _ptr(oh, ctypes.c_int32), _ptr(orr, ctypes.c_int32),
                                 _ptr(ot, ctypes.c_int32), _ptr(od, ctypes.c_double))
        if total < 0:
            raise ValueError("oracle rejected its arguments (p must be 1 or 2)")
        if total <= cap:
            break
        cap = int(total)
    n = int(total)
    oh, orr, ot, od = oh[:n], orr[:n], ot[:n], od[:n]
    order = np.lexsort((ot, oh, orr))
    return {"h": oh[order], "r": orr[order], "t": ot[order], "dist": od[order], "count": n}


def dist_triples(E, Rv, p: int, h, r, t) -> np.ndarray:
    """float64 distances ||E[h] + Rv[r] - E[t]||_p of the listed triples (Section 4.3)."""
    lib = _load()
    E64, R64 = _f64(E), _f64(Rv)
    h = np.ascontiguousarray(h, dtype=np.int32); r = np.ascontiguousarray(r, dtype=np.int32)
    t = np.ascontiguousarray(t, dtype=np.int32)
    if not (h.shape == r.shape == t.shape) or h.ndim != 1:
        raise ValueError("h, r, t must be 1-D arrays of one length")
    if int(p) not in (1, 2):
        raise ValueError("p must be 1 or 2")
    n = h.shape[0]
    if n and (h.min() < 0 or h.max() >= E64.shape[0] or t.min() < 0 or t.max() >= E64.shape[0]
              or r.min() < 0 or r.max() >= R64.shape[0]):
        raise IndexError("triple index out of range")
    out = np.empty(n, np.float64)
    lib.kgco_dist_triples(_ptr(E64, ctypes.c_double), E64.shape[1], _ptr(R64, ctypes.c_double), int(p),
                          _ptr(h, ctypes.c_int32), _ptr(r, ctypes.c_int32), _ptr(t, ctypes.c_int32), n,
                          _ptr(out, ctypes.c_double))
    return out


def top1(E, Rv, p: int, exclude_self: bool = False):
    """The smallest ||E[h] + Rv[r] - E[t]||_p over all triples (the top-1 score of Section 3.3), optionally
    without the self pairs h == t.  Returns a dict h, r, t, dist, or None when no triple is eligible.
    Among equal distances the smallest (r, h, t) is returned."""
    lib = _load()
    E64, R64 = _f64(E), _f64(Rv)
    if int(p) not in (1, 2):
        raise ValueError("p must be 1 or 2")
    if E64.ndim != 2 or R64.ndim != 2 or (E64.shape[0] and R64.shape[0] and E64.shape[1] != R64.shape[1]):
        raise ValueError("E and Rv must be 2-D with one dimension d")
    h, r, t = ctypes.c_int32(-1), ctypes.c_int32(-1), ctypes.c_int32(-1)
    dist = ctypes.c_double(0.0)
    rc = lib.kgco_top1(_ptr(E64, ctypes.c_double), E64.shape[0], E64.shape[1] if E64.shape[0] else R64.shape[1],
                       _ptr(R64, ctypes.c_double), R64.shape[0], int(p), 1 if exclude_self else 0,
                       ctypes.byref(h), ctypes.byref(r), ctypes.byref(t), ctypes.byref(dist))
    if rc < 0:
        raise ValueError("bad argument")
    if rc == 0:
        return None
    return {"h": h.value, "r": r.value, "t": t.value, "dist": dist.value}


def topk(E, Rv, p: int, k: int, exclude_self: bool = False) -> dict:
    """The k triples with the smallest ||E[h] + Rv[r] - E[t]||_p (all eligible ones if there are fewer), ascending
    by (dist, r, h, t): dict of arrays h, r, t, dist and ``count``."""
    lib = _load()
    E64, R64 = _f64(E), _f64(Rv)
    if int(p) not in (1, 2) or k < 0:
        raise ValueError("p must be 1 or 2 and k >= 0")
    k = int(k)
    oh = np.empty(max(k, 1), np.int32); orr = np.empty(max(k, 1), np.int32); ot = np.empty(max(k, 1), np.int32)
    od = np.empty(max(k, 1), np.float64)
    n = lib.kgco_topk(_ptr(E64, ctypes.c_double), E64.shape[0], E64.shape[1] if E64.shape[0] else R64.shape[1],
                      _ptr(R64, ctypes.c_double), R64.shape[0], int(p), 1 if exclude_self else 0, k,
                      _ptr(oh, ctypes.c_int32), _ptr(orr, ctypes.c_int32), _ptr(ot, ctypes.c_int32), _ptr(od, ctypes.c_double))
    if n < 0:
        raise ValueError("bad argument")
    n = int(n)
    return {"h": oh[:n].copy(), "r": orr[:n].copy(), "t": ot[:n].copy(), "dist": od[:n].copy(), "count": n}


def compute_range(sa, sb, eps: float, impl: str = "two_pointer"):
    """Lemma 2: for sorted ``sa``, ``sb`` the first/last j with |sa[i] - sb[j]| <= eps (empty: e = s - 1)."""
    lib = _load()
    sa, sb = _f64(sa), _f64(sb)
    s = np.empty(sa.shape[0], np.int64); e = np.empty(sa.shape[0], np.int64)
    lib.kgco_compute_range(_ptr(sa, ctypes.c_double), sa.shape[0], _ptr(sb, ctypes.c_double), sb.shape[0],
                           float(eps), RANGE_IMPLS[impl], _ptr(s, ctypes.c_int64), _ptr(e, ctypes.c_int64))
    return s, e


def group_ranges(s, e, max_group_size: int):
    """Grouping rule of Section 4.6 for monotone ranges (s_i <= s_{i+1}, e_i <= e_{i+1}).

    Consecutive rows [start, i) are merged into one rectangle
    A'[start:i] x B'[range_min : range_max + 1] while its size
    (range_max - range_min + 1) * (i - start) stays within ``max_group_size``
    (a single row is always accepted).  Returns a list of
    (start, stop, range_min, range_max, size).
    """
    groups = []
    m = len(s)
    start = 0
    while start < m:
        rmin, rmax = int(s[start]), int(e[start])
        i = start + 1
        while i < m:
            nmax = max(rmax, int(e[i]))
            if (nmax - rmin + 1) * (i + 1 - start) > max_group_size:
                break
            rmax = nmax
            i += 1
        groups.append((start, i, rmin, rmax, (rmax - rmin + 1) * (i - start)))
        start = i
    return groups
