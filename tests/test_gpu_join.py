"""GPU parity tests: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest

import oracle
import workloads
from tests import parity

pytestmark = pytest.mark.gpu


def _torch():
    import torch
    return torch


def _dev(x, dtype="f32"):
    torch = _torch()
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16).contiguous() if dtype == "bf16" else t


def _run(E, Rv, p, delta, cap=None, dtype="f32", **kw):
    import paper_2307_12059_amd as kgc
    j = kgc.Join(dtype=dtype, **kw)
    try:
        Ed, Rd = _dev(E, dtype), _dev(Rv, dtype)
        if cap is None:
            cap = 1 << 20
        return j.join(Ed, Rd, p, delta, cap)
    finally:
        j.close()


def _check(E, Rv, p, delta, dtype="f32", **kw):
    """E, Rv: float32 arrays holding the values the device sees."""
    ref = oracle.join(E, Rv, p, delta, mode="abandon")
    got = _run(E, Rv, p, delta, cap=max(1024, 2 * ref["count"]), dtype=dtype, **kw)
    assert got["code"] == 0
    rep = parity.compare(got, ref, E, Rv, p, delta, E.shape[0])
    assert got["count"] == rep["gpu_count"]
    return got, ref, rep


E3 = np.array([[0.0, 0.0], [3.0, 4.0], [1.0, 0.0]], np.float32)
R2 = np.array([[3.0, 4.0], [0.0, 0.0]], np.float32)


@pytest.mark.parametrize("p,delta,count", [(2, 1.0, 7), (2, 5.0, 15), (1, 5.0, 7)])
def test_hand_case(p, delta, count):
    got, ref, rep = _check(E3, R2, p, delta)
    assert got["count"] == count == ref["count"]


PRUNE_OFF, PRUNE_ON = 1, 2


@pytest.mark.parametrize("prune", [PRUNE_OFF, PRUNE_ON])
@pytest.mark.parametrize("tile_cfg", [0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15, 16, 17, 18])
def test_c1_l2_full_parity(tile_cfg, prune):
    if prune == PRUNE_ON and (1 <= tile_cfg <= 5 or tile_cfg >= 15):
        pytest.skip("one-block-per-tile and barrier-free variants have no pruned mode")
    wl = workloads.generate("c1_tiny_l2")
    got, ref, rep = _check(wl.E, wl.Rv, 2, wl.delta, tile_cfg=tile_cfg, prune=prune)
    if prune == PRUNE_ON:
        assert got["stats"]["tiles_pruned"] > 0 and got["stats"]["groups"] > 0
    assert ref["count"] == 3640 and rep["boundary_band"] <= 40
    # the hit decision is taken in double on both sides, so even the boundary band agrees here
    assert rep["only_gpu_in_band"] == 0 and rep["only_oracle_in_band"] == 0
    st = got["stats"]
    assert st["triples_total"] == 2000 * 2000 * 8 and st["emitted"] == got["count"] and st["candidates"] >= got["count"]


@pytest.mark.parametrize("prune", [PRUNE_OFF, PRUNE_ON])
def test_c1_l1_full_parity(prune):
    wl = workloads.generate("c1_tiny_l2")
    h, r, t = workloads.sample_uniform_triples(wl, 200_000, 77)
    delta = float(np.float32(np.sort(oracle.dist_triples(wl.E, wl.Rv, 1, h, r, t))[40]))
    got, ref, rep = _check(wl.E, wl.Rv, 1, delta, prune=prune)
    assert ref["count"] > 1000


@pytest.mark.parametrize("prune", [PRUNE_OFF, PRUNE_ON])
@pytest.mark.parametrize("p", [1, 2])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("N,R,d", [(300, 3, 37), (257, 2, 200), (129, 1, 7), (1, 1, 1), (700, 5, 122),
                                   (600, 3, 300), (300, 2, 960), (520, 2, 218), (520, 2, 219), (400, 2, 282),
                                   (400, 2, 283), (520, 2, 602), (520, 2, 603)])
def test_ragged_shapes(p, dtype, N, R, d, prune):
    g = np.random.default_rng(N * 1000 + d)
    cent = g.standard_normal((4, d))
    E = (cent[g.integers(0, 4, N)] + 0.1 * g.standard_normal((N, d))).astype(np.float32)
    Rv = (cent[g.integers(0, 4, R)] - cent[g.integers(0, 4, R)] + 0.02 * g.standard_normal((R, d))).astype(np.float32)
    if dtype == "bf16":
        E = workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(E))
        Rv = workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(Rv))
    n = min(20000, N * N * R)
    hh, rr, tt = g.integers(0, N, n), g.integers(0, R, n), g.integers(0, N, n)
    delta = float(np.float32(np.quantile(oracle.dist_triples(E, Rv, p, hh, rr, tt), 0.02)))
    got, ref, rep = _check(E, Rv, p, delta, dtype=dtype, prune=prune)
    assert ref["count"] > 0


@pytest.mark.parametrize("prune", [PRUNE_OFF, PRUNE_ON])
@pytest.mark.parametrize("p", [1, 2])
def test_edge_cases(p, prune):
    import paper_2307_12059_amd as kgc
    torch = _torch()
    wl = workloads.generate("c1_tiny_l2", N=400, R=3)
    E, Rv = wl.E, wl.Rv
    # negative threshold and empty inputs: valid, empty
    assert _run(E, Rv, p, -1.0, prune=prune)["count"] == 0
    assert _run(E[:0], Rv, p, 1.0, prune=prune)["count"] == 0
    assert _run(E, Rv[:0], p, 1.0, prune=prune)["count"] == 0
    # zero threshold: only exact coincidences (r = 0 gives the N self pairs)
    assert _run(E, np.zeros_like(Rv[:1]), p, 0.0, prune=prune)["count"] == 400
    # infinite threshold: every triple, each once
    got = _run(E[:70], Rv[:2], p, float("inf"), cap=70 * 70 * 2, prune=prune)
    assert got["count"] == 70 * 70 * 2
    assert np.unique((got["r"].astype(np.int64) * 70 + got["h"]) * 70 + got["t"]).size == 70 * 70 * 2
    np.testing.assert_allclose(got["dist"], oracle.dist_triples(E[:70], Rv[:2], p, got["h"], got["r"], got["t"]),
                               rtol=1e-6)
    # overflow: true count reported, cap valid records, all of them real hits
    ref = oracle.join(E, Rv, p, 3.0 if p == 2 else 14.0)
    assert ref["count"] > 50
    got = _run(E, Rv, p, 3.0 if p == 2 else 14.0, cap=17, prune=prune)
    assert got["code"] == kgc.KGC_OVERFLOW and got["count"] == ref["count"] and got["h"].size == 17
    refset = set(zip(ref["r"].tolist(), ref["h"].tolist(), ref["t"].tolist()))
    assert all(k in refset for k in zip(got["r"].tolist(), got["h"].tolist(), got["t"].tolist()))
    # cap == 0 with a NULL buffer only counts
    j = kgc.Join(prune=prune)
    rc, cnt = kgc.kgc_join(j.handle, _dev(E).data_ptr(), 400, 32, _dev(Rv).data_ptr(), 3, p,
                           3.0 if p == 2 else 14.0, 0, 0)
    assert rc == kgc.KGC_OVERFLOW and cnt == ref["count"]
    # invalid arguments
    Ed, Rd = _dev(E), _dev(Rv)
    out = torch.empty((16, 4), dtype=torch.int32, device="cuda")
    assert kgc.kgc_join(j.handle, Ed.data_ptr(), 400, 32, Rd.data_ptr(), 3, 3, 1.0, out.data_ptr(), 16)[0] == kgc.KGC_E_INVALID
    assert "p must be" in kgc.kgc_last_error(j.handle)
    assert kgc.kgc_join(j.handle, Ed.data_ptr(), 400, 0, Rd.data_ptr(), 3, p, 1.0, out.data_ptr(), 16)[0] == kgc.KGC_E_INVALID
    assert kgc.kgc_join(j.handle, Ed.data_ptr(), 400, 5000, Rd.data_ptr(), 3, p, 1.0, out.data_ptr(), 16)[0] == kgc.KGC_E_INVALID
    assert kgc.kgc_join(j.handle, 0, 400, 32, Rd.data_ptr(), 3, p, 1.0, out.data_ptr(), 16)[0] == kgc.KGC_E_INVALID
    assert kgc.kgc_join(j.handle, Ed.data_ptr(), 400, 32, Rd.data_ptr(), 3, p, float("nan"), out.data_ptr(), 16)[0] == kgc.KGC_E_INVALID
    assert kgc.kgc_join(j.handle, Ed.data_ptr(), 400, 32, Rd.data_ptr(), 3, p, 1.0, 0, 16)[0] == kgc.KGC_E_INVALID
    assert kgc.kgc_join(j.handle, Ed.data_ptr(), 400, 32, Rd.data_ptr(), 3, p, 1.0, out.data_ptr() + 4, 8)[0] == kgc.KGC_E_INVALID
    j.close()


@pytest.mark.parametrize("prune", [PRUNE_OFF, PRUNE_ON])
def test_zero_relation_symmetry(prune):
    wl = workloads.generate("c1_tiny_l2", N=500, R=1)
    got = _run(wl.E, np.zeros_like(wl.Rv), 2, 0.8, prune=prune)
    S = set(zip(got["h"].tolist(), got["t"].tolist()))
    assert all((t, h) in S for (h, t) in S) and all((i, i) in S for i in range(500))


def test_repeatable_and_tile_independent():
    wl = workloads.generate("c1_tiny_l2", N=1500, R=4)
    ref = None
    for tile_cfg, prune in ((1, 1), (1, 1), (2, 1), (6, 1), (8, 1), (10, 1), (11, 1), (13, 1), (9, 2), (9, 2), (10, 2), (0, 2)):
        got = _run(wl.E, wl.Rv, 2, 0.7, tile_cfg=tile_cfg, prune=prune)
        key = np.sort((got["r"].astype(np.int64) * 1500 + got["h"]) * 1500 + got["t"])
        assert ref is None or np.array_equal(ref, key)
        ref = key


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_kernel1_norms(dtype):
    import paper_2307_12059_amd as kgc
    wl = workloads.generate("c1_tiny_l2", N=333, R=3, d=45)
    E, Rv = wl.E, wl.Rv
    if dtype == "bf16":
        E = workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(E)); Rv = workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(Rv))
    j = kgc.Join(dtype=dtype)
    nB, nA = j.norms(_dev(E, dtype), _dev(Rv, dtype))
    j.close()
    rb = lambda x: workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(x.astype(np.float32))).astype(np.float64)
    refB = (rb(E) ** 2).sum(1)
    refA = np.stack([(rb(E + Rv[r]) ** 2).sum(1) for r in range(3)])
    np.testing.assert_allclose(nB.cpu().numpy(), refB, rtol=2e-6)
    np.testing.assert_allclose(nA.cpu().numpy(), refA, rtol=2e-6)
    # zero pivot (Section 4.5): sqrt(nB) is distB up to the bf16 rounding of the operand
    np.testing.assert_allclose(np.sqrt(nB.cpu().numpy()), np.linalg.norm(E.astype(np.float64), axis=1), rtol=5e-3)


# ---- relation-factorised dense L2 join (optional mode): same result set as every other path ----
def test_factorised_hand_case():
    for delta, count in ((1.0, 7), (5.0, 15)):
        got, ref, rep = _check(E3, R2, 2, delta, prune=PRUNE_OFF, factorised=True)
        assert got["count"] == count == ref["count"]
        assert got["stats"]["join_variant"] == 100


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_factorised_c1_parity(dtype):
    wl = workloads.generate("c1_tiny_l2")
    E, Rv = wl.E, wl.Rv
    if dtype == "bf16":
        E = workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(E))
        Rv = workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(Rv))
    got, ref, rep = _check(E, Rv, 2, wl.delta, dtype=dtype, prune=PRUNE_OFF, factorised=True)
    assert got["stats"]["join_variant"] == 100
    assert rep["only_gpu_in_band"] == 0 and rep["only_oracle_in_band"] == 0
    if dtype == "f32":
        assert ref["count"] == 3640
    # the filter is conservative (no hit lost) and not absurdly loose
    assert got["stats"]["candidates"] >= got["count"]
    assert got["stats"]["candidates"] <= 50 * max(1, got["count"])


@pytest.mark.parametrize("N,R,d", [(300, 3, 37), (257, 70, 200), (129, 1, 7), (1, 1, 1), (700, 5, 122), (400, 2, 282),
                                   (400, 2, 283)])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_factorised_ragged_shapes(dtype, N, R, d):
    g = np.random.default_rng(N * 1000 + d + 7)
    cent = g.standard_normal((4, d))
    E = (cent[g.integers(0, 4, N)] + 0.1 * g.standard_normal((N, d))).astype(np.float32)
    Rv = (cent[g.integers(0, 4, R)] - cent[g.integers(0, 4, R)] + 0.02 * g.standard_normal((R, d))).astype(np.float32)
    if dtype == "bf16":
        E = workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(E))
        Rv = workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(Rv))
    delta = 0.1 * np.sqrt(2.0 * d) * 1.05
    got, ref, rep = _check(E, Rv, 2, float(np.float32(delta)), dtype=dtype, prune=PRUNE_OFF, factorised=True)
    # d = 283 does not fit the head-resident tile: the library then takes its ordinary dense kernel
    assert got["stats"]["join_variant"] == (100 if d <= 282 else 17)
    assert rep["only_gpu_in_band"] == 0 and rep["only_oracle_in_band"] == 0


# ---- top-1 score (Section 3.3): smallest triple distance, with and without self pairs ----
def _top1(E, Rv, p, exclude_self, dtype="f32", **kw):
    import paper_2307_12059_amd as kgc
    j = kgc.Join(dtype=dtype, **kw)
    try:
        return j.top1(_dev(E, dtype), _dev(Rv, dtype), p, exclude_self)
    finally:
        j.close()


def _check_top1(E, Rv, p, exclude_self, dtype="f32", **kw):
    ref = oracle.top1(E, Rv, p, exclude_self)
    got = _top1(E, Rv, p, exclude_self, dtype=dtype, **kw)
    if ref is None:
        assert got is None
        return got, ref
    assert got is not None
    # the distance is unique; the triple is checked to attain it (several triples may tie within float precision)
    tol = max(1e-6 * ref["dist"], 1e-6)
    assert abs(got["dist"] - ref["dist"]) <= tol
    dg = oracle.dist_triples(E, Rv, p, [got["h"]], [got["r"]], [got["t"]])[0]
    assert abs(dg - ref["dist"]) <= tol
    if exclude_self:
        assert got["h"] != got["t"]
    return got, ref


def test_top1_hand_case():
    Z = np.zeros((1, 2), np.float32)
    for p in (1, 2):
        for prune in (PRUNE_OFF, PRUNE_ON):
            got, ref = _check_top1(E3, R2, p, False, prune=prune)
            assert (got["r"], got["h"], got["t"]) == (0, 0, 1) == (ref["r"], ref["h"], ref["t"])
            got, ref = _check_top1(E3, R2, p, True, prune=prune)
            assert (got["r"], got["h"], got["t"]) == (0, 0, 1)
            got, ref = _check_top1(E3, Z, p, False, prune=prune)
            assert (got["r"], got["h"], got["t"], got["dist"]) == (0, 0, 0, 0.0)
            got, ref = _check_top1(E3, Z, p, True, prune=prune)
            assert (got["r"], got["h"], got["t"], got["dist"]) == (0, 0, 2, 1.0)
    assert _top1(E3[:1], R2, 2, True) is None                       # one entity: only self pairs
    one = _top1(E3[:1], R2, 2, False)                               # the self pair under the zero relation
    assert (one["r"], one["h"], one["t"], one["dist"]) == (1, 0, 0, 0.0)
    assert _top1(E3[:1], R2[:1], 2, False)["dist"] == pytest.approx(5.0)


@pytest.mark.parametrize("exclude_self", [False, True])
@pytest.mark.parametrize("prune", [PRUNE_OFF, PRUNE_ON])
@pytest.mark.parametrize("p", [1, 2])
def test_top1_c1(p, prune, exclude_self):
    wl = workloads.generate("c1_tiny_l2")
    _check_top1(wl.E, wl.Rv, p, exclude_self, prune=prune)


@pytest.mark.parametrize("exclude_self", [False, True])
def test_top1_with_self_edges_and_overflow(exclude_self):
    # a zero relation makes every self pair a zero-distance triple; duplicated rows make far more than the
    # inner buffer of 2^20 records qualify at the first threshold, so the search has to shrink it
    g = np.random.default_rng(5)
    base = g.standard_normal((40, 16)).astype(np.float32)
    E = np.repeat(base, 60, axis=0)                                   # 2400 rows, 60 copies of each
    Rv = np.concatenate([np.zeros((1, 16), np.float32), g.standard_normal((2, 16)).astype(np.float32)])
    got, ref = _check_top1(E, Rv, 2, exclude_self, prune=PRUNE_ON)
    assert ref["dist"] == 0.0 and got["dist"] == 0.0


# ---- relation ranges (the relation-wise partition of Section 4.7): the union of the parts is the whole ----
@pytest.mark.parametrize("mode", ["dense", "prune", "factorised", "l1"])
def test_join_range_partition(mode):
    import paper_2307_12059_amd as kgc
    wl = workloads.generate("c1_tiny_l2")
    p = 1 if mode == "l1" else 2
    delta = wl.delta if p == 2 else 2.6
    ref = oracle.join(wl.E, wl.Rv, p, delta, mode="abandon")
    assert ref["count"] > 0
    j = kgc.Join(prune=PRUNE_ON if mode in ("prune", "l1") else PRUNE_OFF, factorised=(mode == "factorised"))
    try:
        Ed, Rd = _dev(wl.E, "f32"), _dev(wl.Rv, "f32")
        R = wl.Rv.shape[0]
        parts = []
        for lo, hi in ((0, 3), (3, 3), (3, 4), (4, R)):              # an empty range among them
            got = j.join(Ed, Rd, p, delta, 1 << 16, r_range=(lo, hi))
            assert got["code"] == 0
            assert np.all((got["r"] >= lo) & (got["r"] < hi))
            assert got["count"] == int(np.sum((ref["r"] >= lo) & (ref["r"] < hi)))
            assert got["stats"]["triples_total"] == wl.E.shape[0] ** 2 * (hi - lo)
            parts.append(got)
        merged = {k: np.concatenate([g[k] for g in parts]) for k in ("h", "r", "t", "dist")}
        rep = parity.compare(merged, ref, wl.E, wl.Rv, p, delta, wl.E.shape[0])
        assert rep["gpu_count"] == ref["count"] and rep["only_gpu_in_band"] == 0 and rep["only_oracle_in_band"] == 0
        # a range whose result does not fit reports the overflow with the true count of the range
        small = j.join(Ed, Rd, p, delta, 8, r_range=(0, R))
        assert small["code"] == 1 and small["count"] == ref["count"]
        with pytest.raises(RuntimeError):
            j.join(Ed, Rd, p, delta, 8, r_range=(2, R + 1))
    finally:
        j.close()


# ---- general form of Section 4.3: connector outputs supplied by the caller (kgc_join_ab) ----
def _run_ab(A, B, p, delta, cap, dtype="f32", prune=PRUNE_OFF):
    import paper_2307_12059_amd as kgc
    torch = _torch()
    def dev(x):
        t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()
        return t.to(torch.bfloat16).contiguous() if dtype == "bf16" else t
    j = kgc.Join(dtype=dtype, prune=prune)
    try:
        return j.join_ab(dev(A), dev(B), p, delta, cap)
    finally:
        j.close()


def _compare_ab(got, ref, A, B, p, delta, N):
    """Set equality outside the boundary band, distances to 1e-4 (the TransE comparison on (r, h, t) keys)."""
    per_rel = B.ndim == 3
    def dist(h, r, t):
        x = A[r, h].astype(np.float64) - (B[r, t] if per_rel else B[t]).astype(np.float64)
        return np.sqrt((x * x).sum(-1)) if p == 2 else np.abs(x).sum(-1)
    gk = (got["r"].astype(np.int64) * N + got["h"]) * N + got["t"]
    rk = (ref["r"].astype(np.int64) * N + ref["h"]) * N + ref["t"]
    assert np.unique(gk).size == gk.size
    tol = parity.BAND * abs(delta)
    only_g, only_r = ~np.isin(gk, rk), ~np.isin(rk, gk)
    if only_g.any():
        dg = dist(got["h"][only_g], got["r"][only_g], got["t"][only_g])
        assert np.all(np.abs(dg - delta) <= tol), "GPU triples outside the oracle set and outside the band"
    assert np.all(np.abs(ref["dist"][only_r] - delta) <= tol), "oracle triples missing outside the band"
    go, ro = np.argsort(gk), np.argsort(rk)
    cg, cr = np.isin(gk[go], rk), np.isin(rk[ro], gk)
    dg, dr = got["dist"][go][cg].astype(np.float64), ref["dist"][ro][cr]
    assert np.all(np.abs(dg - dr) <= np.maximum(parity.DIST_RTOL * np.abs(dr), parity.DIST_ATOL))
    return int(only_g.sum()), int(only_r.sum())


@pytest.mark.parametrize("prune", [PRUNE_OFF, PRUNE_ON])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("p", [1, 2])
@pytest.mark.parametrize("N,R,d", [(300, 3, 37), (520, 2, 200), (260, 2, 300), (200, 2, 700), (1500, 5, 64)])
def test_join_ab_structured_embedding(p, dtype, N, R, d, prune):
    """Relation-dependent connectors on both sides (the structured-embedding model of Section 4.3)."""
    g = np.random.default_rng(N + d + p)
    cent = g.standard_normal((4, d))
    E = (cent[g.integers(0, 4, N)] + 0.1 * g.standard_normal((N, d))).astype(np.float32)
    W1 = (np.eye(d) + 0.05 * g.standard_normal((R, d, d)) / np.sqrt(d)).astype(np.float32)
    W2 = (np.eye(d) + 0.05 * g.standard_normal((R, d, d)) / np.sqrt(d)).astype(np.float32)
    A = np.einsum("rij,nj->rni", W1, E).astype(np.float32)
    B = np.einsum("rij,nj->rni", W2, E).astype(np.float32)
    if dtype == "bf16":
        A = workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(A)).reshape(A.shape)
        B = workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(B)).reshape(B.shape)
    # a threshold that keeps pairs of one cluster, about 1 % of all
    probe = np.sqrt(((A[0, :64, None, :] - B[0, None, :64, :]) ** 2).sum(-1)) if p == 2 else np.abs(A[0, :64, None, :] - B[0, None, :64, :]).sum(-1)
    delta = float(np.float32(np.quantile(probe, 0.05)))
    ref = oracle.join_ab(A, B, p, delta)
    assert ref["count"] > 0
    got = _run_ab(A, B, p, delta, max(1024, 2 * ref["count"]), dtype=dtype, prune=prune)
    assert got["code"] == 0
    _compare_ab(got, ref, A, B, p, delta, N)
    if prune == PRUNE_OFF:
        assert got["stats"]["join_variant"] == (0 if p == 1 else 18 if d <= 282 else 17 if d <= 602 else 9)
    else:
        assert got["stats"]["join_variant"] == (0 if p == 1 else 14 if d <= 250 else 9)
        assert got["stats"]["groups"] > 0
        if N >= 1500:
            assert got["stats"]["tiles_pruned"] > 0


@pytest.mark.parametrize("prune", [PRUNE_OFF, PRUNE_ON])
@pytest.mark.parametrize("p", [1, 2])
def test_join_ab_is_transe_on_its_connectors(p, prune):
    """A[r][h] = E[h] + Rv[r] (formed in float32), B = E shared: the same triples as kgc_join up to the rounding of A."""
    wl = workloads.generate("c1_tiny_l2")
    delta = wl.delta if p == 2 else 2.6
    A = (wl.E[None, :, :] + wl.Rv[:, None, :]).astype(np.float32)
    ref = oracle.join_ab(A, wl.E, p, delta)
    got = _run_ab(A, wl.E, p, delta, max(1024, 2 * ref["count"]), prune=prune)
    assert got["code"] == 0 and ref["count"] > 0
    _compare_ab(got, ref, A, wl.E, p, delta, wl.E.shape[0])
    if prune == PRUNE_ON:
        assert got["stats"]["tiles_pruned"] > 0
    base = oracle.join(wl.E, wl.Rv, p, delta, mode="abandon")
    assert abs(got["count"] - base["count"]) <= 5
    # overflow and empty inputs follow kgc_join's conventions
    small = _run_ab(A, wl.E, p, delta, 8, prune=prune)
    assert small["code"] == 1 and small["count"] == got["count"]
    assert _run_ab(A, wl.E, p, -1.0, 8, prune=prune)["count"] == 0


# ---- top-k: the k smallest triple distances ----
def _check_topk(E, Rv, p, k, exclude_self, **kw):
    import paper_2307_12059_amd as kgc
    ref = oracle.topk(E, Rv, p, k, exclude_self)
    j = kgc.Join(**kw)
    try:
        got = j.topk(_dev(E, "f32"), _dev(Rv, "f32"), p, k, exclude_self)
    finally:
        j.close()
    assert got["count"] == ref["count"]
    # the distances are unique (as a sorted list); which of several equal-distance triples come back is not
    assert np.allclose(got["dist"], ref["dist"], rtol=1e-6, atol=1e-6)
    key = (got["r"].astype(np.int64) * E.shape[0] + got["h"]) * E.shape[0] + got["t"]
    assert np.unique(key).size == key.size
    dg = oracle.dist_triples(E, Rv, p, got["h"], got["r"], got["t"])
    assert np.allclose(np.sort(dg), ref["dist"], rtol=1e-6, atol=1e-6)
    if exclude_self:
        assert np.all(got["h"] != got["t"])
    return got, ref


@pytest.mark.parametrize("exclude_self", [False, True])
@pytest.mark.parametrize("p", [1, 2])
def test_topk_hand_case(p, exclude_self):
    for k in (1, 2, 5, 18, 40):                       # 18 triples in all (12 without the self pairs)
        got, ref = _check_topk(E3, R2, p, k, exclude_self)
        assert got["count"] == min(k, 12 if exclude_self else 18)


@pytest.mark.parametrize("prune", [PRUNE_OFF, PRUNE_ON])
@pytest.mark.parametrize("k", [1, 10, 1000, 20000])
def test_topk_c1(k, prune):
    wl = workloads.generate("c1_tiny_l2")
    _check_topk(wl.E, wl.Rv, 2, k, False, prune=prune)
    if k <= 1000:
        _check_topk(wl.E, wl.Rv, 1, k, True, prune=prune)


def test_topk_mass_ties():
    g = np.random.default_rng(5)
    base = g.standard_normal((40, 16)).astype(np.float32)
    E = np.repeat(base, 60, axis=0)
    Rv = np.concatenate([np.zeros((1, 16), np.float32), g.standard_normal((2, 16)).astype(np.float32)])
    for excl in (False, True):
        got, ref = _check_topk(E, Rv, 2, 5000, excl, prune=PRUNE_ON)      # 144,000 zero-distance triples
        assert np.all(got["dist"] == 0.0)


@pytest.mark.parametrize("prune", [PRUNE_OFF, PRUNE_ON])
def test_topk_per_relation(prune):
    """kgc_topk_range with a range of one relation: the k best (h, t) pairs of that relation."""
    import paper_2307_12059_amd as kgc
    wl = workloads.generate("c1_tiny_l2")
    j = kgc.Join(prune=prune)
    try:
        Ed, Rd = _dev(wl.E, "f32"), _dev(wl.Rv, "f32")
        for r in (0, 3, wl.Rv.shape[0] - 1):
            for k, excl in ((1, False), (50, True)):
                got = j.topk(Ed, Rd, 2, k, excl, r_range=(r, r + 1))
                ref = oracle.topk(wl.E, wl.Rv[r:r + 1], 2, k, excl)
                assert got["count"] == ref["count"] == k
                assert np.all(got["r"] == r)
                assert np.allclose(got["dist"], ref["dist"], rtol=1e-6, atol=1e-6)
                dg = oracle.dist_triples(wl.E, wl.Rv, 2, got["h"], got["r"], got["t"])
                assert np.allclose(np.sort(dg), ref["dist"], rtol=1e-6, atol=1e-6)
        assert j.topk(Ed, Rd, 2, 5, r_range=(2, 2))["count"] == 0
        with pytest.raises(RuntimeError):
            j.topk(Ed, Rd, 2, 5, r_range=(0, wl.Rv.shape[0] + 1))
    finally:
        j.close()


@pytest.mark.parametrize("p", [1, 2])
def test_block_pairs_through_the_general_form(p):
    """The partition-based join of Section 4.7: entities cut into blocks, every (head block, tail block) pair joined
    on its own through kgc_join_ab (A = head block + r, B = tail block), indices shifted by the block offsets.
    The union is the join of the whole (the float32 rounding of A stays far inside the boundary band)."""
    wl = workloads.generate("c1_tiny_l2")
    E, Rv = wl.E[:900], wl.Rv
    delta = wl.delta if p == 2 else 2.6
    ref = oracle.join(E, Rv, p, delta, mode="abandon")
    assert ref["count"] > 0
    nb = 300
    parts = {k: [] for k in ("h", "r", "t", "dist")}
    for h0 in range(0, 900, nb):
        A = (E[None, h0:h0 + nb, :] + Rv[:, None, :]).astype(np.float32)
        for t0 in range(0, 900, nb):
            got = _run_ab(A, E[t0:t0 + nb], p, delta, 1 << 16)
            assert got["code"] == 0
            parts["h"].append(got["h"] + h0); parts["t"].append(got["t"] + t0)
            parts["r"].append(got["r"]); parts["dist"].append(got["dist"])
    merged = {k: np.concatenate(v) for k, v in parts.items()}
    rep = parity.compare(merged, ref, E, Rv, p, delta, 900)
    assert rep["gpu_count"] + rep["only_oracle_in_band"] >= ref["count"] - rep["boundary_band"]


@pytest.mark.parametrize("p", [1, 2])
def test_pruning_with_a_threshold_far_below_the_cluster_size(p):
    """A small delta must not switch the pruning off: the group radius is widened until groups form."""
    g = np.random.default_rng(3)
    cent = 4.0 * g.standard_normal((12, 48))
    E = (cent[g.integers(0, 12, 3000)] + 0.3 * g.standard_normal((3000, 48))).astype(np.float32)
    Rv = (cent[g.integers(0, 12, 5)] - cent[g.integers(0, 12, 5)]).astype(np.float32)
    # members of a cluster are about 0.3 * sqrt(2 * 48) = 2.9 apart (L2); the threshold is a small fraction of that
    delta = 0.4 if p == 2 else 2.0
    got, ref, rep = _check(E, Rv, p, delta, prune=PRUNE_ON)
    st = got["stats"]
    assert st["tiles_pruned"] >= 0.8 * st["tiles_total"], st
    assert rep["only_gpu_in_band"] == 0 and rep["only_oracle_in_band"] == 0
