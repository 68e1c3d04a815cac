"""Seeded synthetic inputs for the TransE similarity join.

This module is the only code shared by the CPU oracle's tests and the GPU path's
tests/bench.  It draws random numbers and converts storage formats; it evaluates
no triple distance and takes no join decision.  The thresholds in
``deltas.json`` are *inputs* like the embeddings: they were written by
``oracle/select_delta.py`` (which calls only the oracle) and are read back here.

The five workloads stand in for the LibKGE TransE embeddings the paper measures
on (Section 5.1: FB15K has 14,951 entities and 1,345 relation types, WN18RR has
40,943 entities and 11 relation types; model dimensions 128-512).  Those
checkpoints are not available, so entities are drawn from Gaussian mixtures with
the same shapes and with a threshold larger than a coordinate range (Section 3.3).
"""
from __future__ import annotations

import json
import os
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
DELTAS_PATH = os.path.join(_HERE, "deltas.json")


@dataclass(frozen=True)
class WorkloadSpec:
    """Shape and distribution of one synthetic workload."""

    name: str
    index: int            # position in the benchmark's config list (seed = 1000 + index)
    N: int                # entities
    R: int                # relation vectors
    d: int                # embedding dimension
    K: int                # Gaussian clusters
    sigma: float          # within-cluster standard deviation
    rel_noise: float      # std of the noise added to centre differences (0 = none)
    p: int                # norm of the join: 1 or 2
    storage: str          # "f32" or "bf16"
    selectivity: float    # target fraction of the N*N*R triples that qualify
    zipf: float = 0.0     # >0: cluster sizes proportional to rank**-zipf
    delta_rule: str = "aligned"   # "uniform" (C1) or "aligned" (C2..C5)

    @property
    def seed(self) -> int:
        return 1000 + self.index

    @property
    def n_triples(self) -> int:
        return self.N * self.N * self.R


SPECS = {
    "c1_tiny_l2": WorkloadSpec("c1_tiny_l2", 0, 2_000, 8, 32, 20, 0.1, 0.02, 2, "f32", 1e-4,
                               delta_rule="uniform"),
    "c2_mid_l2": WorkloadSpec("c2_mid_l2", 1, 15_000, 1_345, 100, 500, 0.15, 0.02, 2, "f32", 1e-6),
    "c3_l1": WorkloadSpec("c3_l1", 2, 40_000, 18, 100, 200, 0.1, 0.02, 1, "f32", 1e-6),
    "c4_large_l2": WorkloadSpec("c4_large_l2", 3, 100_000, 200, 200, 2_000, 0.1, 0.0, 2, "bf16", 1e-7),
    "c5_scale_l2": WorkloadSpec("c5_scale_l2", 4, 1_000_000, 1_000, 128, 10_000, 0.05, 0.02, 2, "bf16",
                                1e-9, zipf=1.1),
}


@dataclass
class Workload:
    """One generated instance.

    ``E`` and ``Rv`` hold the values the join sees: float32 arrays for "f32"
    storage; for "bf16" storage they are float32 arrays whose values are exactly
    representable in bfloat16, and ``E_bits`` / ``Rv_bits`` hold the 16-bit
    patterns that go to the device.
    """

    spec: WorkloadSpec
    E: np.ndarray
    Rv: np.ndarray
    labels: np.ndarray          # cluster of each entity, int32[N]
    rel_src: np.ndarray         # cluster i of each relation (r = c_j - c_i + noise), int32[R]
    rel_dst: np.ndarray         # cluster j of each relation, int32[R]
    E_bits: Optional[np.ndarray] = None
    Rv_bits: Optional[np.ndarray] = None
    delta: Optional[float] = None
    meta: dict = field(default_factory=dict)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round to nearest, ties to even); returns uint16 bit patterns.

    Finite inputs only (the generator never produces NaN or infinity).
    """
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _cluster_sizes(spec: WorkloadSpec, N: int, K: int) -> Optional[np.ndarray]:
    if spec.zipf <= 0.0:
        return None
    w = np.arange(1, K + 1, dtype=np.float64) ** (-spec.zipf)
    sizes = np.maximum(1, np.floor(w / w.sum() * N)).astype(np.int64)
    # hand the rounding remainder to the largest clusters, one entity each
    rem = N - int(sizes.sum())
    i = 0
    while rem != 0:
        step = 1 if rem > 0 else -1
        if sizes[i % K] + step >= 1:
            sizes[i % K] += step
            rem -= step
        i += 1
    return sizes


def generate(name: str, *, N: Optional[int] = None, R: Optional[int] = None, d: Optional[int] = None,
             K: Optional[int] = None, seed: Optional[int] = None, with_delta: bool = True) -> Workload:
    """Generate workload ``name``; the keyword overrides make scaled-down variants for tests.

    All draws are float64 from ``numpy.random.Generator(PCG64(seed))`` with one
    spawned sub-stream each for centres, assignment, entity noise, relation
    pairs and relation noise; values are then cast to float32 (and rounded to
    bfloat16 for "bf16" storage).
    """
    spec = SPECS[name]
    N = spec.N if N is None else int(N)
    R = spec.R if R is None else int(R)
    d = spec.d if d is None else int(d)
    K = spec.K if K is None else int(K)
    seed = spec.seed if seed is None else int(seed)
    scaled = (N, R, d, K, seed) != (spec.N, spec.R, spec.d, spec.K, spec.seed)

    ss = np.random.SeedSequence(seed)
    s_cent, s_assign, s_noise, s_pairs, s_rnoise = [np.random.Generator(np.random.PCG64(s)) for s in ss.spawn(5)]

    centres = s_cent.standard_normal((K, d))
    sizes = _cluster_sizes(spec, N, K)
    if sizes is None:
        labels = s_assign.integers(0, K, size=N).astype(np.int32)
    else:
        labels = np.repeat(np.arange(K, dtype=np.int32), sizes)
        s_assign.shuffle(labels)

    E = np.empty((N, d), dtype=np.float32)
    chunk = 65536
    for lo in range(0, N, chunk):
        hi = min(N, lo + chunk)
        E[lo:hi] = (centres[labels[lo:hi]] + spec.sigma * s_noise.standard_normal((hi - lo, d))).astype(np.float32)

    src = s_pairs.integers(0, K, size=R).astype(np.int32)
    off = s_pairs.integers(1, K, size=R).astype(np.int32) if K > 1 else np.zeros(R, dtype=np.int32)
    dst = ((src + off) % K).astype(np.int32)          # distinct from src whenever K > 1
    Rv64 = centres[dst] - centres[src]
    if spec.rel_noise > 0.0:
        Rv64 = Rv64 + spec.rel_noise * s_rnoise.standard_normal((R, d))
    Rv = Rv64.astype(np.float32)

    wl = Workload(spec=spec, E=E, Rv=Rv, labels=labels, rel_src=src, rel_dst=dst)
    if spec.storage == "bf16":
        wl.E_bits = f32_to_bf16_bits(E)
        wl.Rv_bits = f32_to_bf16_bits(Rv)
        wl.E = bf16_bits_to_f32(wl.E_bits)
        wl.Rv = bf16_bits_to_f32(wl.Rv_bits)
    wl.meta = {"N": N, "R": R, "d": d, "K": K, "seed": seed, "scaled": scaled}

    if with_delta and not scaled:
        wl.delta = stored_delta(name)
    return wl


def stored_delta(name: str) -> Optional[float]:
    """Threshold of the full-size workload, as written by ``oracle/select_delta.py`` (a float32 value)."""
    if not os.path.exists(DELTAS_PATH):
        return None
    with open(DELTAS_PATH) as f:
        table = json.load(f)
    ent = table.get(name)
    return None if ent is None else float(np.float32(ent["delta"]))


def sample_uniform_triples(wl: Workload, n: int, seed: int):
    """``n`` triples (h, r, t) drawn uniformly from E x R x E."""
    g = np.random.Generator(np.random.PCG64(seed))
    N, R = wl.E.shape[0], wl.Rv.shape[0]
    return (g.integers(0, N, size=n).astype(np.int32), g.integers(0, R, size=n).astype(np.int32),
            g.integers(0, N, size=n).astype(np.int32))


def aligned_triple_count(wl: Workload) -> int:
    """Number of triples whose head lies in the relation's source cluster and tail in its target cluster."""
    sizes = np.bincount(wl.labels, minlength=int(max(wl.rel_src.max(), wl.rel_dst.max())) + 1).astype(np.int64)
    return int((sizes[wl.rel_src] * sizes[wl.rel_dst]).sum())


def sample_aligned_triples(wl: Workload, n: int, seed: int):
    """``n`` triples drawn uniformly from the aligned triples (see ``aligned_triple_count``)."""
    g = np.random.Generator(np.random.PCG64(seed))
    Kmax = int(max(wl.labels.max(), wl.rel_src.max(), wl.rel_dst.max())) + 1
    sizes = np.bincount(wl.labels, minlength=Kmax).astype(np.int64)
    order = np.argsort(wl.labels, kind="stable").astype(np.int64)
    start = np.concatenate([[0], np.cumsum(sizes)[:-1]])
    w = (sizes[wl.rel_src] * sizes[wl.rel_dst]).astype(np.float64)
    if w.sum() <= 0:
        raise ValueError("no aligned triples in this workload")
    r = g.choice(wl.Rv.shape[0], size=n, p=w / w.sum()).astype(np.int32)
    ci, cj = wl.rel_src[r], wl.rel_dst[r]
    h = order[start[ci] + (g.random(n) * sizes[ci]).astype(np.int64)]
    t = order[start[cj] + (g.random(n) * sizes[cj]).astype(np.int64)]
    return h.astype(np.int32), r, t.astype(np.int32)


def cluster_aligned_subsample(wl: Workload, n_rel: int, max_entities: int, seed: int):
    """Pick ``n_rel`` relations and the entities of the clusters they link (at most ``max_entities`` in total).

    Returns (entity_ids, relation_ids), both sorted.  A join restricted to these
    ids contains aligned triples, so a brute-force check on it is not vacuous.
    """
    g = np.random.Generator(np.random.PCG64(seed))
    R = wl.Rv.shape[0]
    rel = np.sort(g.choice(R, size=min(n_rel, R), replace=False)).astype(np.int32)
    clusters = np.unique(np.concatenate([wl.rel_src[rel], wl.rel_dst[rel]]))
    # every linked cluster keeps an equal share of the budget, so that skewed cluster sizes cannot crowd
    # the small clusters (and with them the aligned triples) out of the sample
    per_cluster = max(1, max_entities // max(1, clusters.size))
    parts = []
    for c in clusters:
        members = np.nonzero(wl.labels == c)[0]
        if members.size > per_cluster:
            members = g.choice(members, size=per_cluster, replace=False)
        parts.append(members)
    ent = np.sort(np.concatenate(parts)) if parts else np.empty(0, np.int64)
    return ent.astype(np.int32), rel
