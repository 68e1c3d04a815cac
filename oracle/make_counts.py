"""Full-size reference sets of the synthetic workloads, reduced to what a test can carry.

Runs the oracle's early-abandon mode (pinned to brute force by tests/test_oracle_pins.py) over the whole
workload and stores, per workload, in tests/golden/oracle_counts.json:
  count            number of qualifying triples
  band             triples with |dist - delta| <= 1e-4 * delta, listed explicitly as [r, h, t]
  digest_no_band   SHA-256 over the sorted keys (r * N + h) * N + t (little-endian int64) of the set
                   with the band triples removed
Calls only the oracle and the input generator.  Run from the repo root:
    python -m oracle.make_counts c2_mid_l2 c3_l1 ...
The mid workload takes about a quarter of an hour on 8 cores, the large one a few hours.
"""
from __future__ import annotations

import hashlib
import json
import os
import sys
import time

import numpy as np

import oracle
import workloads

OUT = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "tests", "golden", "oracle_counts.json")
BAND = 1e-4


def digest(keys: np.ndarray) -> str:
    return hashlib.sha256(np.sort(np.asarray(keys, np.int64)).astype("<i8").tobytes()).hexdigest()


def reference(name: str) -> dict:
    wl = workloads.generate(name)
    spec = wl.spec
    t0 = time.time()
    res = oracle.join(wl.E, wl.Rv, spec.p, wl.delta, mode="abandon", cap=int(8 * spec.selectivity * spec.n_triples) + 4096)
    N = spec.N
    keys = (res["r"].astype(np.int64) * N + res["h"]) * N + res["t"]
    band = np.abs(res["dist"] - wl.delta) <= BAND * wl.delta
    return {"count": int(res["count"]), "band": [[int(r), int(h), int(t)] for r, h, t in
                                                  zip(res["r"][band], res["h"][band], res["t"][band])],
            "digest_no_band": digest(keys[~band]), "delta": wl.delta, "p": spec.p, "N": N, "R": spec.R, "d": spec.d,
            "seconds": round(time.time() - t0, 1), "threads": oracle.num_threads()}


def main(argv):
    try:
        with open(OUT) as f:
            table = json.load(f)
    except FileNotFoundError:
        table = {}
    for name in argv:
        table[name] = reference(name)
        print(name, {k: v for k, v in table[name].items() if k != "band"}, "band triples:", len(table[name]["band"]), flush=True)
        with open(OUT, "w") as f:
            json.dump(table, f, indent=1, sort_keys=True)
            f.write("\n")


if __name__ == "__main__":
    main(sys.argv[1:])
