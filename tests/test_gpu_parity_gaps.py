"""GPU parity on inputs the benchmark workloads do not have: embeddings far from the origin, embeddings without
cluster structure under pruning, arrays that start off a 16-byte boundary, joins cut into several relation batches
by a small workspace, an exact-stage block list that has to grow, and a seeded sweep over random shapes, norms,
storage types and modes.  Every case is compared with the CPU oracle, set against set (tests/parity.py)."""
import os

import numpy as np
import pytest

import oracle
import workloads
from tests import parity

pytestmark = pytest.mark.gpu

PRUNE_OFF, PRUNE_ON = 1, 2


def _seen(x, dtype):
    """The float32 values the device sees for storage type `dtype`."""
    x = np.ascontiguousarray(x, np.float32)
    if dtype == "bf16":
        return workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(x)).reshape(x.shape)
    return x


def _dev(x, dtype, offset=0):
    """x (values already representable in `dtype`) on the device, `offset` elements past an aligned address."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x, np.float32)).cuda()
    if dtype == "bf16":
        t = t.to(torch.bfloat16)
    if offset:
        buf = torch.empty(t.numel() + offset + 8, dtype=t.dtype, device="cuda")
        assert buf.data_ptr() % 256 == 0
        view = buf[offset:offset + t.numel()].view(t.shape)
        view.copy_(t)
        assert view.is_contiguous() and view.data_ptr() % 16 != 0
        return view
    return t.contiguous()


def _clustered(g, N, R, d, K, sig, shift=0.0):
    cent = g.standard_normal((K, d))
    E = cent[g.integers(0, K, N)] + sig * g.standard_normal((N, d)) + shift
    Rv = cent[g.integers(0, K, R)] - cent[g.integers(0, K, R)] + 0.02 * g.standard_normal((R, d))
    return E.astype(np.float32), Rv.astype(np.float32)


def _join_and_compare(E, Rv, p, delta, dtype, offset=(0, 0), **kw):
    import paper_2307_12059_amd as kgc
    ref = oracle.join(E, Rv, p, delta, mode="abandon")
    j = kgc.Join(dtype=dtype, **kw)
    try:
        got = j.join(_dev(E, dtype, offset[0]), _dev(Rv, dtype, offset[1]), p, delta, max(1024, 2 * ref["count"]))
    finally:
        j.close()
    assert got["code"] == 0
    rep = parity.compare(got, ref, E, Rv, p, delta, E.shape[0])
    return got, ref, rep


# ---- embeddings far from the origin: the norms are large against the distances, so the expansion
# ---- ||a||^2 + ||b||^2 - 2 a.b cancels almost everything and the bound test works on large centre norms
@pytest.mark.parametrize("prune", [PRUNE_OFF, PRUNE_ON])
@pytest.mark.parametrize("p", [1, 2])
@pytest.mark.parametrize("dtype,shift", [("f32", 40.0), ("f32", 400.0), ("bf16", 6.0)])
def test_translated_embeddings(p, dtype, shift, prune):
    g = np.random.default_rng(1000 + p + int(shift))
    N, R, d, sig = 1400, 4, 100, 0.1
    E, Rv = _clustered(g, N, R, d, 9, sig, shift=shift)
    Rv[0] = 0.0                                        # self pairs qualify at distance 0 whatever the shift
    E, Rv = _seen(E, dtype), _seen(Rv, dtype)
    delta = float(np.float32(sig * np.sqrt(2.0 * d) * 1.0 if p == 2 else sig * np.sqrt(2.0) * d * 0.8))
    if dtype == "bf16":                                # bf16 at |x| ~ 6 has a spacing of 1/32: the clusters smear out
        delta *= 1.3
    got, ref, rep = _join_and_compare(E, Rv, p, delta, dtype, prune=prune)
    assert ref["count"] >= N, "vacuous: not even the self pairs"
    assert rep["gpu_count"] == got["count"]


# ---- no cluster structure: the grouping finds nothing to group, the bound test must still be safe
@pytest.mark.parametrize("p", [1, 2])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("d", [16, 100])
def test_unclustered_embeddings_with_pruning(p, dtype, d):
    g = np.random.default_rng(2000 + d + p)
    N, R = 1500, 3
    E = _seen(g.standard_normal((N, d)), dtype)
    Rv = _seen(0.3 * g.standard_normal((R, d)), dtype)
    # delta: a low quantile of the distances of sampled triples, so that hits exist but are rare
    h, t, r = g.integers(0, N, 200000), g.integers(0, N, 200000), g.integers(0, R, 200000)
    x = E[h].astype(np.float64) + Rv[r] - E[t]
    dist = np.sqrt((x * x).sum(-1)) if p == 2 else np.abs(x).sum(-1)
    delta = float(np.float32(np.quantile(dist[h != t], 2e-4)))
    got, ref, rep = _join_and_compare(E, Rv, p, delta, dtype, prune=PRUNE_ON)
    assert ref["count"] > 50
    dense, _, _ = _join_and_compare(E, Rv, p, delta, dtype, prune=PRUNE_OFF)
    assert dense["count"] == got["count"] or rep["boundary_band"] > 0


# ---- arrays that start 1 .. 3 elements past a 16-byte boundary (the vector loads of the exact path must not be used)
@pytest.mark.parametrize("mode", ["dense", "prune", "factorised"])
@pytest.mark.parametrize("p", [1, 2])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("offset", [(1, 0), (0, 3), (3, 1)])
def test_unaligned_arrays(p, dtype, offset, mode):
    if mode == "factorised" and p == 1:
        pytest.skip("the relation-factorised form is L2 only")
    g = np.random.default_rng(3000 + 10 * offset[0] + offset[1] + p)
    N, R, d, sig = 900, 3, 100, 0.1                    # d = 100: rows are 16-byte multiples, only the base is off
    E, Rv = _clustered(g, N, R, d, 6, sig)
    E, Rv = _seen(E, dtype), _seen(Rv, dtype)
    delta = float(np.float32(sig * np.sqrt(2.0 * d) if p == 2 else sig * np.sqrt(2.0) * d * 0.8))
    got, ref, rep = _join_and_compare(E, Rv, p, delta, dtype, offset=offset,
                                      prune=PRUNE_ON if mode == "prune" else PRUNE_OFF, factorised=(mode == "factorised"))
    assert ref["count"] > 100


@pytest.mark.parametrize("exclude_self", [False, True])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_unaligned_arrays_top1_and_topk(dtype, exclude_self):
    import paper_2307_12059_amd as kgc
    g = np.random.default_rng(3100)
    N, R, d = 700, 3, 100
    E, Rv = _clustered(g, N, R, d, 6, 0.1)
    E, Rv = _seen(E, dtype), _seen(Rv, dtype)
    j = kgc.Join(dtype=dtype, prune=PRUNE_ON)
    try:
        Ed, Rd = _dev(E, dtype, 1), _dev(Rv, dtype, 3)
        t1 = j.top1(Ed, Rd, 2, exclude_self)
        tk = j.topk(Ed, Rd, 2, 50, exclude_self)
    finally:
        j.close()
    o1 = oracle.top1(E, Rv, 2, exclude_self)
    ok = oracle.topk(E, Rv, 2, 50, exclude_self)
    assert abs(t1["dist"] - o1["dist"]) <= 1e-6 * max(o1["dist"], 1.0)
    np.testing.assert_allclose(np.sort(tk["dist"]), np.sort(ok["dist"]), rtol=1e-6, atol=1e-6)


# ---- a small workspace cuts the relations into several batches
@pytest.mark.parametrize("mode", ["dense", "prune", "factorised"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_relation_batches_from_a_small_workspace(mode, dtype):
    g = np.random.default_rng(4000)
    N, R, d, sig = 700, 7, 122, 0.1
    E, Rv = _clustered(g, N, R, d, 5, sig)
    E, Rv = _seen(E, dtype), _seen(Rv, dtype)
    delta = float(np.float32(sig * np.sqrt(2.0 * d)))
    # one relation's staged operands: 4 K slices x 768 rows x 64 bytes = 192 KiB; the factorised form keeps
    # 768 x 4 bytes per relation
    ws = 3 * 768 * 4 if mode == "factorised" else 2 * (4 * 768 * 64 + 768 * 4) + 1000
    got, ref, rep = _join_and_compare(E, Rv, 2, delta, dtype, workspace_bytes=ws,
                                      prune=PRUNE_ON if mode == "prune" else PRUNE_OFF, factorised=(mode == "factorised"))
    assert got["stats"]["relation_batches"] >= 3, got["stats"]
    assert ref["count"] > 100


@pytest.mark.parametrize("per_rel", [False, True])
@pytest.mark.parametrize("prune", [PRUNE_OFF, PRUNE_ON])
@pytest.mark.parametrize("p", [1, 2])
def test_relation_batches_general_form(p, prune, per_rel):
    import paper_2307_12059_amd as kgc
    if p == 1 and prune == PRUNE_OFF:
        pytest.skip("the dense L1 join stages nothing per relation: no workspace limit cuts it")
    g = np.random.default_rng(4100 + p)
    N, R, d, sig = 600, 6, 64, 0.1
    E, _ = _clustered(g, N, R, d, 5, sig)
    W1 = (np.eye(d) + 0.03 * g.standard_normal((R, d, d)) / np.sqrt(d)).astype(np.float32)
    A = np.einsum("rij,nj->rni", W1, E).astype(np.float32)
    if per_rel:
        W2 = (np.eye(d) + 0.03 * g.standard_normal((R, d, d)) / np.sqrt(d)).astype(np.float32)
        B = np.einsum("rij,nj->rni", W2, E).astype(np.float32)
    else:
        B = E.copy()
    delta = float(np.float32(sig * np.sqrt(2.0 * d) if p == 2 else sig * np.sqrt(2.0) * d * 0.8))
    ref = oracle.join_ab(A, B, p, delta)
    # p = 2: 3 K slices x 640 rows x 64 bytes per relation and operand; p = 1 (pruned): centres of 20 micro-tiles
    ws = 2 * (3 * 640 * 64) * (2 if per_rel else 1) + 100 if p == 2 else 2 * (20 * d * 4 * 2) + 100
    j = kgc.Join(dtype="f32", prune=prune, workspace_bytes=ws)
    try:
        got = j.join_ab(_dev(A, "f32"), _dev(B, "f32"), p, delta, max(1024, 2 * ref["count"]))
    finally:
        j.close()
    assert got["code"] == 0 and got["stats"]["relation_batches"] >= 3, got["stats"]
    gk = (got["r"].astype(np.int64) * N + got["h"]) * N + got["t"]
    rk = (ref["r"].astype(np.int64) * N + ref["h"]) * N + ref["t"]
    assert np.unique(gk).size == gk.size
    og, orr = ~np.isin(gk, rk), ~np.isin(rk, gk)
    tol = parity.BAND * abs(delta)
    if og.any():
        x = A[got["r"][og], got["h"][og]].astype(np.float64) - (B[got["r"][og], got["t"][og]] if per_rel else B[got["t"][og]])
        dg = np.sqrt((x * x).sum(-1)) if p == 2 else np.abs(x).sum(-1)
        assert np.all(np.abs(dg - delta) <= tol)
    assert np.all(np.abs(ref["dist"][orr] - delta) <= tol)
    assert ref["count"] > 100


# ---- the block list of the exact stage starts too short and has to grow (the join then runs again)
@pytest.mark.parametrize("prune", [PRUNE_OFF, PRUNE_ON])
def test_exact_block_list_grows(prune):
    wl = workloads.generate("c1_tiny_l2")
    normal, ref, _ = _join_and_compare(wl.E, wl.Rv, 2, wl.delta, "f32", prune=prune, tile_cfg=14)
    os.environ["KGC_EXACT_LIST_CAP"] = "3"
    try:
        small, _, _ = _join_and_compare(wl.E, wl.Rv, 2, wl.delta, "f32", prune=prune, tile_cfg=14)
    finally:
        del os.environ["KGC_EXACT_LIST_CAP"]
    assert normal["stats"]["exact_blocks"] > 3
    assert small["count"] == normal["count"] == ref["count"]
    if prune == PRUNE_OFF:       # (the grouping of a pruned join may differ from run to run, and the blocks with it)
        assert small["stats"]["exact_blocks"] == normal["stats"]["exact_blocks"]
        assert small["stats"]["candidates"] == normal["stats"]["candidates"]
    else:
        assert small["stats"]["exact_blocks"] > 3


# ---- the barrier-free kernel walking tile lists (the pruned default for many entities, here chosen by hand): whole
# ---- lists in the LDS, and lists cut into segments of two entries
@pytest.mark.parametrize("segment", [0, 2])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_pruned_barrier_free_kernel_walks_tile_lists(segment, dtype):
    g = np.random.default_rng(515 + segment)
    N, R, d, sig = 3000, 5, 64, 0.1
    E, Rv = _clustered(g, N, R, d, 4, sig)               # four clusters of 750: rows with several surviving 256 x 256 tiles
    E, Rv = _seen(E, dtype), _seen(Rv, dtype)
    delta = float(np.float32(sig * np.sqrt(2.0 * d) * 0.9))
    if segment:
        os.environ["KGC_TILE_LIST_SEGMENT"] = str(segment)
    try:
        got, ref, _ = _join_and_compare(E, Rv, 2, delta, dtype, prune=PRUNE_ON, tile_cfg=15)
    finally:
        os.environ.pop("KGC_TILE_LIST_SEGMENT", None)
    assert got["stats"]["join_variant"] == 15
    assert ref["count"] > 0


# ---- the tile-at-a-time kernel with so few workgroups that each walks several batches of tiles (its list entries are
# ---- staged per batch of 32 tiles, the flagged blocks listed per batch)
def test_tile_at_a_time_kernel_walks_several_batches():
    g = np.random.default_rng(616)
    N, R, d, sig = 2600, 24, 64, 0.1
    E, Rv = _clustered(g, N, R, d, 40, sig)              # 40 clusters of 65: a surviving tile or two per (relation, head tile)
    delta = float(np.float32(sig * np.sqrt(2.0 * d) * 0.8))
    normal, ref, _ = _join_and_compare(E, Rv, 2, delta, "f32", prune=PRUNE_ON)
    os.environ["KGC_PAIRS_GRID"] = "2"
    try:
        few, _, _ = _join_and_compare(E, Rv, 2, delta, "f32", prune=PRUNE_ON)
    finally:
        del os.environ["KGC_PAIRS_GRID"]
    tiles = normal["stats"]["tiles_total"] - normal["stats"]["tiles_pruned"]
    assert tiles > 2 * 32 * 2, f"vacuous: {tiles} surviving tiles do not make two batches for each of two workgroups"
    assert few["count"] == normal["count"] == ref["count"] > 0


# ---- seeded sweep: random shapes (ragged in N and d, through every kernel family's range of d), cluster widths,
# ---- norms, storage types, thresholds and modes; bounded so that the oracle side stays within a minute
def _fuzz_cases(seed, n):
    g = np.random.default_rng(seed)
    for case in range(n):
        N = int(g.integers(1, 2500)); R = int(g.integers(1, 12))
        d = int(g.choice([3, 17, 32, 64, 100, 128, 200, 218, 219, 250, 251, 282, 283, 400, 602, 603, 700]))
        K = int(g.integers(1, 10)); sig = float(g.choice([0.05, 0.1, 0.3]))
        p = int(g.choice([1, 2])); dtype = str(g.choice(["f32", "bf16"]))
        mode = str(g.choice(["dense", "prune", "factorised"])) if p == 2 else str(g.choice(["dense", "prune"]))
        scale = float(g.choice([0.6, 0.9, 1.0, 1.1, 1.5]))
        yield case, g, N, R, d, K, sig, p, dtype, mode, scale


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_seeded_sweep_join(seed):
    import paper_2307_12059_amd as kgc
    for case, g, N, R, d, K, sig, p, dtype, mode, scale in _fuzz_cases(seed, 30):
        E, Rv = _clustered(g, N, R, d, K, sig)
        E, Rv = _seen(E, dtype), _seen(Rv, dtype)
        base = sig * np.sqrt(2.0 * d) if p == 2 else sig * np.sqrt(2.0) * d * 0.8
        delta = float(np.float32(base * scale))
        print(f"seed {seed} case {case}: N={N} R={R} d={d} K={K} p={p} {dtype} {mode} delta={delta:.4g}", flush=True)
        ref = oracle.join(E, Rv, p, delta, mode="abandon")
        if ref["count"] > 1_500_000:
            continue
        j = kgc.Join(dtype=dtype, prune=PRUNE_ON if mode == "prune" else PRUNE_OFF, factorised=(mode == "factorised"))
        try:
            Ed, Rd = _dev(E, dtype), _dev(Rv, dtype)
            got = j.join(Ed, Rd, p, delta, max(1024, 2 * ref["count"]))
            assert got["code"] == 0
            parity.compare(got, ref, E, Rv, p, delta, N)
            if ref["count"] > 0 and case % 3 == 0:
                t1 = j.top1(Ed, Rd, p, bool(case % 2))
                o1 = oracle.top1(E, Rv, p, bool(case % 2))
                assert (t1 is None) == (o1 is None)
                if o1:
                    assert abs(t1["dist"] - o1["dist"]) <= 1e-6 * max(o1["dist"], 1.0), (t1, o1)
        finally:
            j.close()


@pytest.mark.parametrize("seed", [21, 22])
def test_seeded_sweep_general_form(seed):
    import paper_2307_12059_amd as kgc
    g = np.random.default_rng(seed)
    for case in range(16):
        N = int(g.integers(1, 1800)); R = int(g.integers(1, 6)); d = int(g.choice([5, 32, 64, 100, 200, 219, 300]))
        K = int(g.integers(1, 10)); sig = float(g.choice([0.05, 0.1, 0.3]))
        p = int(g.choice([1, 2])); dtype = str(g.choice(["f32", "bf16"]))
        per_rel = bool(g.integers(0, 2)); prune = bool(g.integers(0, 2))
        E, _ = _clustered(g, N, R, d, K, sig)
        W1 = (np.eye(d) + 0.03 * g.standard_normal((R, d, d)) / np.sqrt(d)).astype(np.float32)
        A = np.einsum("rij,nj->rni", W1, E).astype(np.float32)
        if per_rel:
            W2 = (np.eye(d) + 0.03 * g.standard_normal((R, d, d)) / np.sqrt(d)).astype(np.float32)
            B = np.einsum("rij,nj->rni", W2, E).astype(np.float32)
        else:
            B = E.copy()
        A, B = _seen(A, dtype), _seen(B, dtype)
        base = sig * np.sqrt(2.0 * d) if p == 2 else sig * np.sqrt(2.0) * d * 0.8
        delta = float(np.float32(base * float(g.choice([0.3, 0.9, 1.0, 1.2]))))
        print(f"seed {seed} case {case}: N={N} R={R} d={d} p={p} {dtype} per_rel={per_rel} prune={prune} delta={delta:.4g}", flush=True)
        ref = oracle.join_ab(A, B, p, delta)
        if ref["count"] > 1_500_000:
            continue
        j = kgc.Join(dtype=dtype, prune=PRUNE_ON if prune else PRUNE_OFF)
        try:
            got = j.join_ab(_dev(A, dtype), _dev(B, dtype), p, delta, max(1024, 2 * ref["count"]))
        finally:
            j.close()
        assert got["code"] == 0
        gk = (got["r"].astype(np.int64) * N + got["h"]) * N + got["t"]
        rk = (ref["r"].astype(np.int64) * N + ref["h"]) * N + ref["t"]
        assert np.unique(gk).size == gk.size
        og, orr = ~np.isin(gk, rk), ~np.isin(rk, gk)
        tol = parity.BAND * abs(delta)
        if og.any():
            x = A[got["r"][og], got["h"][og]].astype(np.float64) - (B[got["r"][og], got["t"][og]] if per_rel else B[got["t"][og]])
            dg = np.sqrt((x * x).sum(-1)) if p == 2 else np.abs(x).sum(-1)
            assert np.all(np.abs(dg - delta) <= tol), "a GPU triple the definition rejects, outside the band"
        assert np.all(np.abs(ref["dist"][orr] - delta) <= tol), "a qualifying triple is missing, outside the band"


# ---- the structured-embedding instance (Section 4.3): connectors formed on the device, oracle on float64 connectors
def _se_case(g, N, R, d, sig, dtype):
    E, _ = _clustered(g, N, R, d, 6, sig)
    W1 = (np.eye(d) + 0.03 * g.standard_normal((R, d, d)) / np.sqrt(d)).astype(np.float32)
    W2 = (np.eye(d) + 0.03 * g.standard_normal((R, d, d)) / np.sqrt(d)).astype(np.float32)
    E, W1, W2 = _seen(E, dtype), _seen(W1, dtype), _seen(W2, dtype)
    # the connector rows in double, from the values the device sees: a_{r,h} = W1[r] h, b_{r,t} = W2[r] t
    A = np.einsum("rij,nj->rni", W1.astype(np.float64), E.astype(np.float64))
    B = np.einsum("rij,nj->rni", W2.astype(np.float64), E.astype(np.float64))
    return E, W1, W2, A, B


@pytest.mark.parametrize("prune", [PRUNE_OFF, PRUNE_ON])
@pytest.mark.parametrize("p", [1, 2])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("N,R,d,ws", [(700, 5, 64, 0), (300, 3, 37, 0), (520, 7, 200, 4 * 3 * 520 * 200 * 4)])
def test_structured_embedding_join(p, dtype, N, R, d, ws, prune):
    import paper_2307_12059_amd as kgc
    g = np.random.default_rng(5000 + p + d)
    sig = 0.1
    E, W1, W2, A, B = _se_case(g, N, R, d, sig, dtype)
    delta = float(np.float32(sig * np.sqrt(2.0 * d) if p == 2 else sig * np.sqrt(2.0) * d * 0.8))
    ref = oracle.join_ab(A, B, p, delta)
    assert ref["count"] > 100
    j = kgc.Join(dtype=dtype, prune=prune, workspace_bytes=ws)
    try:
        got = j.join_se(_dev(E, dtype), _dev(W1, dtype), _dev(W2, dtype), p, delta, max(1024, 2 * ref["count"]))
    finally:
        j.close()
    assert got["code"] == 0
    if ws:
        assert got["stats"]["relation_batches"] >= 3     # the connector buffers held three relations at a time
    gk = (got["r"].astype(np.int64) * N + got["h"]) * N + got["t"]
    rk = (ref["r"].astype(np.int64) * N + ref["h"]) * N + ref["t"]
    assert np.unique(gk).size == gk.size == got["count"]
    og, orr = ~np.isin(gk, rk), ~np.isin(rk, gk)
    tol = parity.BAND * abs(delta)       # float32 connector rounding (about 1e-5 of a distance here) stays inside it
    if og.any():
        x = A[got["r"][og], got["h"][og]] - B[got["r"][og], got["t"][og]]
        dg = np.sqrt((x * x).sum(-1)) if p == 2 else np.abs(x).sum(-1)
        assert np.all(np.abs(dg - delta) <= tol), "a GPU triple the definition rejects, outside the band"
    assert np.all(np.abs(ref["dist"][orr] - delta) <= tol), "a qualifying triple is missing, outside the band"
    # reported distances against the float64 connectors
    x = A[got["r"], got["h"]] - B[got["r"], got["t"]]
    dref = np.sqrt((x * x).sum(-1)) if p == 2 else np.abs(x).sum(-1)
    np.testing.assert_allclose(got["dist"], dref, rtol=parity.DIST_RTOL, atol=parity.DIST_ATOL)


def test_structured_embedding_join_overflow_and_empty():
    import paper_2307_12059_amd as kgc
    import torch
    g = np.random.default_rng(5100)
    N, R, d = 300, 4, 32
    E, W1, W2, A, B = _se_case(g, N, R, d, 0.1, "f32")
    delta = float(np.float32(0.1 * np.sqrt(2.0) * d * 0.8))
    ref = oracle.join_ab(A, B, 1, delta)
    j = kgc.Join(dtype="f32", workspace_bytes=4 * 2 * N * d * 4)       # two relations per connector batch
    try:
        got = j.join_se(_dev(E, "f32"), _dev(W1, "f32"), _dev(W2, "f32"), 1, delta, 50)
        assert got["code"] == kgc.KGC_OVERFLOW and got["count"] == ref["count"] and got["h"].size == 50
        rk = set(((ref["r"].astype(np.int64) * N + ref["h"]) * N + ref["t"]).tolist())
        gk = ((got["r"].astype(np.int64) * N + got["h"]) * N + got["t"]).tolist()
        assert len(set(gk)) == 50 and all(k in rk for k in gk)       # (no band triples at this seed)
        none = j.join_se(_dev(E, "f32"), torch.empty((0, d, d), device="cuda"), torch.empty((0, d, d), device="cuda"), 1, delta, 10)
        assert none["code"] == 0 and none["count"] == 0
    finally:
        j.close()


# ---- the join block by block with a cursor (Section 4.7): a small buffer is drained again and again
def _drain_blocks(j, Ed, Rd, p, delta, cap, block_rows, rel_block, max_calls=10000):
    import paper_2307_12059_amd as kgc
    parts, cursor, calls = [], None, 0
    while True:
        got = j.join_blocks(Ed, Rd, p, delta, cap, block_rows, rel_block, cursor)
        cursor = got["cursor"]
        calls += 1
        assert calls <= max_calls
        if got["code"] == kgc.KGC_OVERFLOW and got["count"] == 0:
            assert cursor.need > cap          # one unit alone is larger than the buffer: take a larger one for it
            cap = int(cursor.need)
            continue
        parts.append(got)
        if got["code"] == 0:
            assert cursor.unit == cursor.units
            break
        assert got["code"] == kgc.KGC_OVERFLOW and 0 < cursor.need
    out = {k: np.concatenate([q[k] for q in parts]) for k in ("h", "r", "t", "dist")}
    out["count"] = int(out["h"].size)
    return out, calls, cursor


@pytest.mark.parametrize("prune", [PRUNE_OFF, PRUNE_ON])
@pytest.mark.parametrize("p", [1, 2])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("N,block_rows,rel_block", [(1100, 256, 2), (700, 300, 5), (1300, 1024, 1)])
def test_join_blocks_drains_to_the_oracle_set(p, dtype, N, block_rows, rel_block, prune):
    import paper_2307_12059_amd as kgc
    g = np.random.default_rng(6000 + N + p)
    R, d, sig = 5, 64, 0.1
    E, Rv = _clustered(g, N, R, d, 7, sig)
    E, Rv = _seen(E, dtype), _seen(Rv, dtype)
    delta = float(np.float32(sig * np.sqrt(2.0 * d) if p == 2 else sig * np.sqrt(2.0) * d * 0.8))
    ref = oracle.join(E, Rv, p, delta, mode="abandon")
    assert ref["count"] > 1000
    j = kgc.Join(dtype=dtype, prune=prune)
    try:
        got, calls, cursor = _drain_blocks(j, _dev(E, dtype), _dev(Rv, dtype), p, delta, max(64, ref["count"] // 7), block_rows, rel_block)
    finally:
        j.close()
    assert calls >= 3, "the buffer was meant to be too small for one call"
    nb = -(-(-(-N // 256) * 256) // (-(-block_rows // 256) * 256))
    assert cursor.units >= (-(-R // rel_block)) * nb * nb          # (a grouped order may pad itself into more blocks)
    parity.compare(got, ref, E, Rv, p, delta, N)                   # set against set, every triple once


def test_join_blocks_equals_join_in_one_call_and_survives_other_calls():
    import paper_2307_12059_amd as kgc
    g = np.random.default_rng(6100)
    N, R, d, sig = 900, 4, 37, 0.1
    E, Rv = _clustered(g, N, R, d, 5, sig)
    delta = float(np.float32(sig * np.sqrt(2.0 * d)))
    ref = oracle.join(E, Rv, 2, delta, mode="abandon")
    Ed, Rd = _dev(E, "f32"), _dev(Rv, "f32")
    # everything in one call when the buffer is large enough
    j = kgc.Join(dtype="f32", prune=PRUNE_ON)
    try:
        got = j.join_blocks(Ed, Rd, 2, delta, 2 * ref["count"], 512, 2)
        assert got["code"] == 0 and got["cursor"].unit == got["cursor"].units
        parity.compare(got, ref, E, Rv, 2, delta, N)
        # a pruned join that is continued after another call on the handle is refused, not silently wrong
        first = j.join_blocks(Ed, Rd, 2, delta, max(64, ref["count"] // 5), 512, 2)
        assert first["code"] == kgc.KGC_OVERFLOW and first["cursor"].unit > 0
        j.top1(Ed, Rd, 2)
        with pytest.raises(RuntimeError, match="row order"):
            j.join_blocks(Ed, Rd, 2, delta, max(64, ref["count"] // 5), 512, 2, first["cursor"])
    finally:
        j.close()
    # a dense join keeps going: its row order is the entity order
    j = kgc.Join(dtype="f32", prune=PRUNE_OFF)
    try:
        cap = max(64, ref["count"] // 5)
        parts, cursor = [], None
        for step in range(1000):
            got = j.join_blocks(Ed, Rd, 2, delta, cap, 512, 2, cursor)
            cursor = got["cursor"]
            if got["code"] == kgc.KGC_OVERFLOW and got["count"] == 0:
                cap = int(cursor.need)
                continue
            parts.append(got)
            if got["code"] == 0:
                break
            j.top1(Ed, Rd, 2)               # the handle is used for something else between the calls
        allp = {k: np.concatenate([q[k] for q in parts]) for k in ("h", "r", "t", "dist")}
        allp["count"] = int(allp["h"].size)
        parity.compare(allp, ref, E, Rv, 2, delta, N)
    finally:
        j.close()


def test_join_blocks_edge_cases():
    import paper_2307_12059_amd as kgc
    import torch
    g = np.random.default_rng(6200)
    N, R, d, sig = 500, 3, 32, 0.1
    E, Rv = _clustered(g, N, R, d, 4, sig)
    delta = float(np.float32(sig * np.sqrt(2.0 * d)))
    ref = oracle.join(E, Rv, 2, delta, mode="abandon")
    Ed, Rd = _dev(E, "f32"), _dev(Rv, "f32")
    for prune in (PRUNE_OFF, PRUNE_ON):
        j = kgc.Join(dtype="f32", prune=prune)
        try:
            # one block, one relation range: a single unit, the same as kgc_join
            one = j.join_blocks(Ed, Rd, 2, delta, 2 * ref["count"], 1 << 20, 1000)
            assert one["code"] == 0 and one["cursor"].units == 1 and one["cursor"].unit == 1
            parity.compare(one, ref, E, Rv, 2, delta, N)
            # no room at all: nothing is returned, the cursor stops at the first unit that has triples and says how many
            none = j.join_blocks(Ed, Rd, 2, delta, 0, 256, 1)
            assert none["code"] == kgc.KGC_OVERFLOW and none["count"] == 0 and none["cursor"].need > 0
            assert none["cursor"].unit < none["cursor"].units
            # a finished cursor: nothing more to do
            done = j.join_blocks(Ed, Rd, 2, delta, 16, 1 << 20, 1000, one["cursor"])
            assert done["code"] == 0 and done["count"] == 0
            # empty inputs
            empty = j.join_blocks(Ed, torch.empty((0, d), device="cuda"), 2, delta, 16, 256, 1)
            assert empty["code"] == 0 and empty["count"] == 0
            empty = j.join_blocks(torch.empty((0, d), device="cuda"), Rd, 2, delta, 16, 256, 1)
            assert empty["code"] == 0 and empty["count"] == 0
            # a negative threshold has no hits in any unit
            neg = j.join_blocks(Ed, Rd, 2, -1.0, 16, 256, 1)
            assert neg["code"] == 0 and neg["count"] == 0 and neg["cursor"].unit == neg["cursor"].units
            with pytest.raises(RuntimeError):
                j.join_blocks(Ed, Rd, 2, delta, 16, 0, 1)
            with pytest.raises(RuntimeError):
                j.join_blocks(Ed, Rd, 2, delta, 16, 256, 0)
        finally:
            j.close()
    j = kgc.Join(dtype="f32", prune=PRUNE_OFF, factorised=True)
    try:
        with pytest.raises(RuntimeError, match="factorised"):
            j.join_blocks(Ed, Rd, 2, delta, 16, 256, 1)
    finally:
        j.close()


def test_many_surviving_tiles_fall_back_to_row_lists():
    """The flat bound test lists the surviving tiles itself when they are few; here nothing can be pruned (no cluster
    structure, 9,000 entities), more than 4,096 tiles survive, and the lists must come from the pass over the bitmap."""
    g = np.random.default_rng(7000)
    N, R, d = 9000, 2, 16
    E = g.standard_normal((N, d)).astype(np.float32)
    Rv = (0.3 * g.standard_normal((R, d))).astype(np.float32)
    h, t, r = g.integers(0, N, 300000), g.integers(0, N, 300000), g.integers(0, R, 300000)
    x = E[h].astype(np.float64) + Rv[r] - E[t]
    dist = np.sqrt((x * x).sum(-1))
    delta = float(np.float32(np.quantile(dist[h != t], 1e-4)))
    got, ref, rep = _join_and_compare(E, Rv, 2, delta, "f32", prune=PRUNE_ON)
    assert ref["count"] > 1000
    assert got["stats"]["tiles_evaluated"] > 4096 and got["stats"]["join_variant"] == 14
