"""Pins for the CPU oracle: everything here is fixed by the paper or by mathematics, not by the oracle itself."""
import itertools
import math
import os

import numpy as np
import pytest
from scipy.spatial.distance import cdist

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")


def _golden():
    out = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, v = [x.strip() for x in line.split("=")]
            vals = [int(x) for x in v.split()]
            out[k] = vals if len(vals) > 1 else vals[0]
    return out


def _set(res):
    return set(zip(res["r"].tolist(), res["h"].tolist(), res["t"].tolist()))


# ---------- hand-computed case (exact in binary) ----------
E3 = np.array([[0.0, 0.0], [3.0, 4.0], [1.0, 0.0]])
R2 = np.array([[3.0, 4.0], [0.0, 0.0]])


@pytest.mark.parametrize("mode", ["brute", "abandon", "pivot"])
def test_hand_case_l2_delta1(mode):
    # r0 = (3,4): e0 + r0 = e1 (dist 0); e2 + r0 - e1 = (1,0) (dist 1).  r1 = 0: selfs, and e0<->e2 at distance 1.
    res = oracle.join(E3, R2, 2, 1.0, mode=mode)
    assert _set(res) == {(0, 0, 1), (0, 2, 1), (1, 0, 0), (1, 0, 2), (1, 1, 1), (1, 2, 0), (1, 2, 2)}
    d = dict(zip(zip(res["r"].tolist(), res["h"].tolist(), res["t"].tolist()), res["dist"].tolist()))
    assert d[(0, 0, 1)] == 0.0 and d[(0, 2, 1)] == 1.0 and d[(1, 0, 2)] == 1.0   # inclusive at exactly delta


@pytest.mark.parametrize("mode", ["brute", "abandon", "pivot"])
def test_hand_case_l2_delta5(mode):
    res = oracle.join(E3, R2, 2, 5.0, mode=mode)
    # r0: (1,0) = 10, (1,2) = sqrt(89), (2,0) = sqrt(32) are out; r1: all nine are in (max is 5)
    expect = {(0, h, t) for h in range(3) for t in range(3)} - {(0, 1, 0), (0, 1, 2), (0, 2, 0)}
    expect |= {(1, h, t) for h in range(3) for t in range(3)}
    assert _set(res) == expect and res["count"] == 15
    d = dict(zip(zip(res["r"].tolist(), res["h"].tolist(), res["t"].tolist()), res["dist"].tolist()))
    assert d[(0, 0, 0)] == 5.0 and d[(0, 0, 2)] == math.sqrt(20.0) and d[(1, 1, 2)] == math.sqrt(20.0)


@pytest.mark.parametrize("mode", ["brute", "abandon", "pivot"])
def test_hand_case_l1_delta5(mode):
    # |(3,4)|_1 = 7 > 5 separates p = 1 from p = 2
    res = oracle.join(E3, R2, 1, 5.0, mode=mode)
    assert _set(res) == {(0, 0, 1), (0, 2, 1), (1, 0, 0), (1, 1, 1), (1, 2, 2), (1, 0, 2), (1, 2, 0)}
    d = dict(zip(zip(res["r"].tolist(), res["h"].tolist(), res["t"].tolist()), res["dist"].tolist()))
    assert d[(0, 2, 1)] == 1.0 and d[(0, 0, 1)] == 0.0


def test_dist_triples_hand_values():
    h = np.array([1, 1, 2, 0], np.int32); r = np.array([0, 0, 0, 1], np.int32); t = np.array([0, 2, 0, 1], np.int32)
    d2 = oracle.dist_triples(E3, R2, 2, h, r, t)
    d1 = oracle.dist_triples(E3, R2, 1, h, r, t)
    assert d2.tolist() == [10.0, math.sqrt(89.0), math.sqrt(32.0), 5.0]
    assert d1.tolist() == [14.0, 13.0, 8.0, 7.0]


# ---------- closed form: points on a line ----------
@pytest.mark.parametrize("p", [1, 2])
@pytest.mark.parametrize("k,m", [(0, 0), (3, 2), (-5, 1), (7, 10)])
def test_lattice_closed_form(p, k, m):
    N, d = 23, 4
    E = np.zeros((N, d)); E[:, 0] = np.arange(N)
    Rv = np.zeros((1, d)); Rv[0, 0] = k
    res = oracle.join(E, Rv, p, float(m))
    # dist(i, j) = |i + k - j|; pairs with i + k - j = s number max(0, N - |k - s|)... counted directly:
    expect = sum(max(0, N - abs(k + s)) for s in range(-m, m + 1))
    assert res["count"] == expect
    assert np.array_equal(res["dist"], np.abs(res["h"] + k - res["t"]).astype(np.float64))


# ---------- library special case: scipy cdist ----------
@pytest.mark.parametrize("p,metric", [(2, "euclidean"), (1, "cityblock")])
def test_matches_cdist(p, metric):
    g = np.random.default_rng(7)
    E = g.standard_normal((60, 9)).astype(np.float32); Rv = (0.3 * g.standard_normal((3, 9))).astype(np.float32)
    full = np.stack([cdist(E.astype(np.float64) + Rv[r].astype(np.float64), E.astype(np.float64), metric)
                     for r in range(3)])
    delta = float(np.quantile(full, 0.05))
    res = oracle.join(E, Rv, p, delta)
    mask = full <= delta
    # cdist may differ from the oracle in the last bits: leave out triples within 1e-12 of the threshold
    band = np.abs(full - delta) <= 1e-12 * delta
    got = np.zeros_like(mask); got[res["r"], res["h"], res["t"]] = True
    assert np.array_equal(got | band, mask | band)
    np.testing.assert_allclose(res["dist"], full[res["r"], res["h"], res["t"]], rtol=1e-13)
    rr, hh, tt = np.nonzero(np.ones_like(mask))
    np.testing.assert_allclose(oracle.dist_triples(E, Rv, p, hh, rr, tt), full.ravel(), rtol=1e-13, atol=1e-15)


# ---------- invariants ----------
def _rand(seed, N=80, R=4, d=6, scale=0.4):
    g = np.random.default_rng(seed)
    return g.standard_normal((N, d)), scale * g.standard_normal((R, d))


@pytest.mark.parametrize("p", [1, 2])
def test_zero_relation_symmetry_and_selfs(p):
    E, _ = _rand(1)
    res = oracle.join(E, np.zeros((1, E.shape[1])), p, 1.5)
    S = _set(res)
    assert all((0, t, h) in S for (_, h, t) in S)
    assert all((0, i, i) in S for i in range(E.shape[0]))
    d = dict(zip(zip(res["h"].tolist(), res["t"].tolist()), res["dist"].tolist()))
    assert all(d[(h, t)] == d[(t, h)] for (h, t) in d)
    assert oracle.join(E, np.zeros((1, E.shape[1])), p, 0.0)["count"] == E.shape[0]


@pytest.mark.parametrize("p", [1, 2])
def test_negation(p):
    E, Rv = _rand(2)
    a = oracle.join(E, Rv, p, 2.0); b = oracle.join(E, -Rv, p, 2.0)
    assert {(r, t, h) for (r, h, t) in _set(a)} == _set(b) and a["count"] > 0


@pytest.mark.parametrize("p", [1, 2])
def test_translation_and_monotone(p):
    E, Rv = _rand(3)
    delta = 2.0
    a = oracle.join(E, Rv, p, delta)
    shift = np.full(E.shape[1], 0.5)            # exact in binary; sums stay exact enough away from the band
    b = oracle.join(E + shift, Rv, p, delta)
    full = oracle.dist_triples(E, Rv, p, *np.array(list(itertools.product(range(80), range(4), range(80))),
                                                    dtype=np.int32).T[[0, 1, 2]])
    assert np.min(np.abs(full - delta)) > 1e-9   # no triple sits on the boundary, so the sets must be equal
    assert _set(a) == _set(b)
    c = oracle.join(E, Rv, p, delta * 0.7)
    assert _set(c) <= _set(a) and c["count"] < a["count"]
    assert oracle.join(E, Rv, p, -1.0)["count"] == 0
    assert oracle.join(E, Rv, p, float("inf"))["count"] == 80 * 80 * 4


def test_norm_ordering():
    E, Rv = _rand(4)
    d = E.shape[1]
    l1 = _set(oracle.join(E, Rv, 1, 2.5)); l2 = _set(oracle.join(E, Rv, 2, 2.5))
    l1_wide = _set(oracle.join(E, Rv, 1, 2.5 * math.sqrt(d)))
    assert l1 <= l2 <= l1_wide and len(l1) < len(l2) < len(l1_wide)


@pytest.mark.parametrize("p", [1, 2])
def test_lemma1_on_every_hit(p):
    """Lemma 1: dist(a, b) >= |dist(p, a) - dist(p, b)| for any pivot."""
    E, Rv = _rand(5)
    res = oracle.join(E, Rv, p, 2.2)
    metric = "euclidean" if p == 2 else "cityblock"
    for pv in (np.zeros(E.shape[1]), E[3], E.mean(0)):
        da = np.stack([cdist(pv[None], E + Rv[r], metric)[0] for r in range(Rv.shape[0])])
        db = cdist(pv[None], E, metric)[0]
        lb = np.abs(da[res["r"], res["h"]] - db[res["t"]])
        assert np.all(lb <= res["dist"] + 1e-12)


@pytest.mark.parametrize("p", [1, 2])
def test_restriction(p):
    E, Rv = _rand(6)
    full = _set(oracle.join(E, Rv, p, 2.0))
    ent = np.array([1, 5, 9, 20, 33, 47, 48, 60, 79]); rel = np.array([0, 3])
    sub = oracle.join(E[ent], Rv[rel], p, 2.0)
    got = {(int(rel[r]), int(ent[h]), int(ent[t])) for (r, h, t) in _set(sub)}
    es, rs = set(ent.tolist()), set(rel.tolist())
    assert got == {(r, h, t) for (r, h, t) in full if r in rs and h in es and t in es}


# ---------- the three modes agree; any pivot gives the same set ----------
@pytest.mark.parametrize("p", [1, 2])
@pytest.mark.parametrize("seed", [11, 12])
def test_modes_agree(p, seed):
    E, Rv = _rand(seed, N=150, R=5, d=12)
    ref = oracle.join(E, Rv, p, 3.0 if p == 2 else 8.0, mode="brute")
    assert ref["count"] > 0
    for mode, kw in [("abandon", {}), ("pivot", {}), ("pivot", {"range_impl": "binary_search"}),
                     ("pivot", {"pivot": E[7]}), ("pivot", {"pivot": E.mean(0)})]:
        got = oracle.join(E, Rv, p, 3.0 if p == 2 else 8.0, mode=mode, **kw)
        assert _set(got) == _set(ref)
        assert np.array_equal(got["dist"], ref["dist"])
        if mode == "pivot":
            assert got["evaluated"] < ref["evaluated"]          # the filter really filters


# ---------- Lemma 2 ----------
def test_compute_range_definition_and_monotone():
    g = np.random.default_rng(21)
    for _ in range(20):
        m, n = int(g.integers(1, 40)), int(g.integers(1, 40))
        sa = np.sort(g.random(m) * 10); sb = np.sort(g.random(n) * 10); eps = float(g.random() * 2)
        s0, e0 = oracle.compute_range(sa, sb, eps, "two_pointer")
        s1, e1 = oracle.compute_range(sa, sb, eps, "binary_search")
        assert np.array_equal(s0, s1) and np.array_equal(e0, e1)
        for i in range(m):                                       # eq. "condition": min / max over the valid j
            ok = np.nonzero(np.abs(sa[i] - sb) <= eps)[0]
            if ok.size:
                assert (s0[i], e0[i]) == (ok.min(), ok.max())
                assert np.all(np.abs(sa[i] - sb[s0[i]:e0[i] + 1]) <= eps)      # eq. "se": the range is contiguous
            else:
                assert e0[i] == s0[i] - 1
        assert np.all(np.diff(s0) >= 0) and np.all(np.diff(e0) >= 0)           # eq. "se2"


def test_compute_range_edges():
    s, e = oracle.compute_range(np.array([]), np.array([1.0]), 1.0)
    assert s.size == 0 and e.size == 0
    s, e = oracle.compute_range(np.array([0.0, 5.0]), np.array([]), 1.0)
    assert s.tolist() == [0, 0] and e.tolist() == [-1, -1]
    s, e = oracle.compute_range(np.array([0.0, 1.0, 2.0]), np.array([1.0, 1.0, 1.0]), 1.0)     # inclusive ends, ties
    assert s.tolist() == [0, 0, 0] and e.tolist() == [2, 2, 2]


# ---------- values the paper prints ----------
def test_paper_grouping_example():
    G = _golden()
    groups = oracle.group_ranges(G["group_s"], G["group_e"], G["max_group_size"])
    assert groups == [(0, G["group_cnt"], G["group_range_min"], G["group_range_max"], G["group_size"])]
    # separate evaluation (Section 4.5): B'[2:5], B'[2:6], B'[4:6] -> 3 + 4 + 2 candidates
    assert [e - s + 1 for s, e in zip(G["group_s"], G["group_e"])] == [3, 4, 2]
    # a budget below the merged size splits the rows again
    assert [g[:2] for g in oracle.group_ranges(G["group_s"], G["group_e"], 8)] == [(0, 2), (2, 3)]


def test_paper_triple_count_is_64bit():
    G = _golden()
    N, R = G["fb15k_entities"], 2 * G["fb15k_relations"]
    assert N * R * N == G["fb15k_triple_scores"]
    # the oracle's own counter: delta = inf on a small case scales the same way
    E = np.zeros((5, 2)); Rv = np.zeros((3, 2))
    res = oracle.join(E, Rv, 2, float("inf"))
    assert res["count"] == res["evaluated"] == 5 * 5 * 3


def test_bad_arguments():
    with pytest.raises(ValueError):
        oracle.join(E3, R2, 3, 1.0)
    with pytest.raises(IndexError):
        oracle.dist_triples(E3, R2, 2, [3], [0], [0])
    assert oracle.join(np.zeros((0, 2)), R2, 2, 1.0)["count"] == 0
    assert oracle.join(E3, np.zeros((0, 2)), 2, 1.0)["count"] == 0


# ---- top-1 score (Section 3.3): the minimum of the triple distance, with and without self pairs ----
def test_top1_hand_case():
    # E3 = {(0,0), (3,4), (1,0)}, R2 = {(3,4), (0,0)}: (h=0, r=0, t=1) has distance 0 and is the smallest (r, h, t)
    # among the zero-distance triples (the others are the self pairs under the zero relation r=1)
    E = np.array([[0.0, 0.0], [3.0, 4.0], [1.0, 0.0]])
    R = np.array([[3.0, 4.0], [0.0, 0.0]])
    for p in (1, 2):
        a = oracle.top1(E, R, p)
        assert (a["r"], a["h"], a["t"]) == (0, 0, 1) and a["dist"] == 0.0
        b = oracle.top1(E, R, p, exclude_self=True)
        assert (b["r"], b["h"], b["t"]) == (0, 0, 1) and b["dist"] == 0.0
    # only the zero relation: every self pair has distance 0; without them the closest pair is (0,0)-(1,0)
    Z = np.zeros((1, 2))
    a = oracle.top1(E, Z, 2)
    assert (a["r"], a["h"], a["t"], a["dist"]) == (0, 0, 0, 0.0)
    b = oracle.top1(E, Z, 2, exclude_self=True)
    assert (b["r"], b["h"], b["t"], b["dist"]) == (0, 0, 2, 1.0)
    b1 = oracle.top1(E, Z, 1, exclude_self=True)
    assert (b1["h"], b1["t"], b1["dist"]) == (0, 2, 1.0)


def test_top1_against_cdist_and_join():
    from scipy.spatial.distance import cdist
    g = np.random.default_rng(77)
    E = g.standard_normal((60, 9)); R = g.standard_normal((4, 9)) * 0.3
    for p, metric in ((2, "euclidean"), (1, "cityblock")):
        D = np.stack([cdist(E + R[r], E, metric) for r in range(R.shape[0])])       # [r][h][t]
        for excl in (False, True):
            Dm = D.copy()
            if excl:
                for r in range(R.shape[0]):
                    np.fill_diagonal(Dm[r], np.inf)
            r, h, t = np.unravel_index(np.argmin(Dm), Dm.shape)
            a = oracle.top1(E, R, p, exclude_self=excl)
            assert (a["r"], a["h"], a["t"]) == (r, h, t)
            assert abs(a["dist"] - Dm[r, h, t]) <= 1e-12 * max(1.0, Dm[r, h, t])
            # the join sees it the same way: nothing below the top-1 distance, the top-1 triple at it
            if not excl:
                below = oracle.join(E, R, p, np.nextafter(a["dist"], -np.inf), mode="brute")
                assert below["count"] == 0
                at = oracle.join(E, R, p, a["dist"], mode="brute")
                assert at["count"] >= 1 and (a["h"], a["r"], a["t"]) in set(zip(at["h"], at["r"], at["t"]))


def test_top1_degenerate():
    E1 = np.ones((1, 3)); R = np.ones((2, 3))
    assert oracle.top1(E1, R, 2, exclude_self=True) is None          # one entity: only self pairs exist
    a = oracle.top1(E1, R, 2)
    assert (a["h"], a["t"]) == (0, 0) and abs(a["dist"] - np.sqrt(3.0)) < 1e-15
    assert oracle.top1(np.zeros((0, 3)), R, 2) is None
    assert oracle.top1(E1, np.zeros((0, 3)), 1) is None


# ---- general form of Section 4.3: connector outputs supplied by the caller ----
def test_join_ab_reduces_to_transe_and_cdist():
    from scipy.spatial.distance import cdist
    g = np.random.default_rng(11)
    E = g.standard_normal((50, 7)); R = g.standard_normal((3, 7)) * 0.4
    A = E[None, :, :] + R[:, None, :]                   # connector_1(h, r) = h + r, connector_2(t, r) = t
    for p, metric, delta in ((2, "euclidean", 2.2), (1, "cityblock", 5.0)):
        ref = oracle.join(E, R, p, delta, mode="brute")
        assert ref["count"] > 0
        for B in (E, E[None], np.broadcast_to(E, (3, 50, 7)).copy()):
            got = oracle.join_ab(A, B, p, delta)
            assert got["count"] == ref["count"]
            assert np.array_equal(got["h"], ref["h"]) and np.array_equal(got["r"], ref["r"]) and np.array_equal(got["t"], ref["t"])
            # (h + r) - t and a - t differ by the rounding of a = h + r only
            assert np.allclose(got["dist"], ref["dist"], rtol=1e-13, atol=1e-13)
    # relation-dependent connector on both sides (SE-like: a = W1_r h, b = W2_r t), against scipy
    W1 = g.standard_normal((3, 7, 7)) * 0.3; W2 = g.standard_normal((3, 7, 7)) * 0.3
    A = np.einsum("rij,nj->rni", W1, E); B = np.einsum("rij,nj->rni", W2, E)
    for p, metric in ((2, "euclidean"), (1, "cityblock")):
        D = np.stack([cdist(A[r], B[r], metric) for r in range(3)])
        delta = float(np.quantile(D, 0.02))
        got = oracle.join_ab(A, B, p, delta)
        rr, hh, tt = np.nonzero(D <= delta)
        assert got["count"] == rr.size > 0
        assert np.array_equal(got["r"], rr) and np.array_equal(got["h"], hh) and np.array_equal(got["t"], tt)
        assert np.allclose(got["dist"], D[rr, hh, tt], rtol=1e-13)
    # a swapped relation index on the B side would show here: B differs per relation
    d2 = float(np.quantile(np.stack([cdist(A[r], B[r]) for r in range(3)]), 0.02))
    straight = oracle.join_ab(A, B, 2, d2)
    swapped = oracle.join_ab(A, B[::-1].copy(), 2, d2)
    assert not (swapped["count"] == straight["count"] and np.array_equal(swapped["h"], straight["h"]))


# ---- top-k: the k smallest triple distances ----
def test_topk_against_sorting_all_distances():
    from scipy.spatial.distance import cdist
    g = np.random.default_rng(19)
    E = g.standard_normal((40, 6)); R = g.standard_normal((3, 6)) * 0.5
    for p, metric in ((2, "euclidean"), (1, "cityblock")):
        D = np.stack([cdist(E + R[r], E, metric) for r in range(3)])        # [r][h][t]
        for excl in (False, True):
            keys = [(D[r, h, t], r, h, t) for r in range(3) for h in range(40) for t in range(40) if not (excl and h == t)]
            keys.sort()
            for k in (1, 7, 100, len(keys) + 5):
                got = oracle.topk(E, R, p, k, exclude_self=excl)
                want = keys[:k]
                assert got["count"] == len(want)
                assert [(r, h, t) for _, r, h, t in want] == list(zip(got["r"], got["h"], got["t"]))
                assert np.allclose(got["dist"], [w[0] for w in want], rtol=1e-13, atol=1e-13)
            one = oracle.top1(E, R, p, exclude_self=excl)
            first = oracle.topk(E, R, p, 1, exclude_self=excl)
            assert (one["r"], one["h"], one["t"]) == (first["r"][0], first["h"][0], first["t"][0])
    assert oracle.topk(E, R, 2, 0)["count"] == 0
    # consistency with the join: the k-th distance as threshold returns at least k triples, all of the top-k among them
    got = oracle.topk(E, R, 2, 25)
    j = oracle.join(E, R, 2, got["dist"][-1], mode="brute")
    assert j["count"] >= 25 and set(zip(got["r"], got["h"], got["t"])) <= set(zip(j["r"], j["h"], j["t"]))
