"""Choose the join threshold of each synthetic workload and store it in workloads/deltas.json.

Calls only the oracle (float64 distances of sampled triples) and the input
generator.  Run from the repo root:  python -m oracle.select_delta [names...]

Rules:
  * "uniform" (the tiny workload): 10^6 uniformly sampled triples; delta is the
    distance below which a fraction ``selectivity`` of them falls (the 100th
    smallest for 1e-4).
  * "aligned" (all others): uniform sampling cannot resolve selectivities of
    1e-6 .. 1e-9, so the sample is drawn from the aligned triples (head in the
    relation's source cluster, tail in its target cluster), which hold nearly
    every hit; delta is their q-quantile with
    q * (#aligned triples) = selectivity * N * N * R.
delta is rounded to float32 once; both the oracle and the GPU use that value.
"""
from __future__ import annotations

import json
import sys

import numpy as np

import oracle
import workloads

N_SAMPLES = {"uniform": 1_000_000, "aligned": 2_000_000}


def select(name: str) -> dict:
    wl = workloads.generate(name, with_delta=False)
    spec = wl.spec
    if spec.delta_rule == "uniform":
        n = N_SAMPLES["uniform"]
        h, r, t = workloads.sample_uniform_triples(wl, n, spec.seed + 500)
        dist = np.sort(oracle.dist_triples(wl.E, wl.Rv, spec.p, h, r, t))
        k = max(1, int(round(spec.selectivity * n)))
        delta64 = dist[k - 1]
        info = {"rule": "uniform", "samples": n, "rank": k}
    else:
        n = N_SAMPLES["aligned"]
        total = workloads.aligned_triple_count(wl)
        q = spec.selectivity * spec.n_triples / total
        if not (0.0 < q < 1.0):
            raise RuntimeError(f"{name}: aligned quantile {q} outside (0, 1)")
        h, r, t = workloads.sample_aligned_triples(wl, n, spec.seed + 500)
        dist = oracle.dist_triples(wl.E, wl.Rv, spec.p, h, r, t)
        delta64 = float(np.quantile(dist, q))
        info = {"rule": "aligned", "samples": n, "aligned_triples": total, "quantile": q}
    delta32 = float(np.float32(delta64))
    info.update({"delta": delta32, "delta_f64": float(delta64), "p": spec.p,
                 "expected_hits": spec.selectivity * spec.n_triples})
    return info


def main(argv):
    names = argv or list(workloads.SPECS)
    try:
        with open(workloads.DELTAS_PATH) as f:
            table = json.load(f)
    except FileNotFoundError:
        table = {}
    for name in names:
        table[name] = select(name)
        print(name, table[name], flush=True)
        with open(workloads.DELTAS_PATH, "w") as f:
            json.dump(table, f, indent=1, sort_keys=True)
            f.write("\n")


if __name__ == "__main__":
    main(sys.argv[1:])
