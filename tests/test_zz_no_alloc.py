"""kgc_join_static -- the entry point that allocates nothing -- against kgc_join (dense), through the C ABI.

Two calls in a row on one handle, the second on a smaller input (the static scratch keeps the first call's
contents), for both norms and both storage types; the result sets must be identical to kgc_join's with
pruning off (bit-exact: same kernels, same exact stage) and also pass the oracle comparison.
"""
import ctypes

import numpy as np
import pytest

import oracle
import workloads
from tests import parity

pytestmark = pytest.mark.gpu


def _dev(x, dtype):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16).contiguous() if dtype == "bf16" else t


def _fetch(out, count, cap):
    host = out[:min(count, cap)].cpu().numpy()
    return {"h": host[:, 0].copy(), "r": host[:, 1].copy(), "t": host[:, 2].copy(), "dist": host[:, 3].copy().view("float32")}


def _sorted(res):
    o = np.lexsort((res["t"], res["h"], res["r"]))
    return res["r"][o], res["h"][o], res["t"][o], res["dist"][o]


def _both(j, kgc, E, Rv, Ed, Rd, p, delta, cap):
    """The same join through kgc_join_static and through kgc_join on a handle with pruning off."""
    import torch
    N, d = E.shape
    R = Rv.shape[0]
    out_s = torch.empty((cap, 4), dtype=torch.int32, device="cuda")
    out_d = torch.empty((cap, 4), dtype=torch.int32, device="cuda")
    rc_s, n_s = kgc.kgc_join_static(j.handle, Ed.data_ptr(), N, d, Rd.data_ptr(), R, p, float(delta), out_s.data_ptr(), cap)
    assert rc_s == kgc.KGC_OK, kgc.kgc_last_error(j.handle)
    st = kgc.kgc_get_stats(j.handle)
    rc_d, n_d = kgc.kgc_join(j.handle, Ed.data_ptr(), N, d, Rd.data_ptr(), R, p, float(delta), out_d.data_ptr(), cap)
    assert rc_d == kgc.KGC_OK
    assert n_s == n_d and n_s <= cap
    got_s, got_d = _fetch(out_s, n_s, cap), _fetch(out_d, n_d, cap)
    for a, b in zip(_sorted(got_s), _sorted(got_d)):
        assert np.array_equal(a, b)                      # same triples, same float distances, bit for bit
    return got_s, st


@pytest.mark.parametrize("p,dtype", [(2, "f32"), (2, "bf16"), (1, "f32"), (1, "bf16")])
def test_static_join_matches_the_allocating_join_twice_in_a_row(p, dtype):
    import paper_2307_12059_amd as kgc
    wl = workloads.generate("c1_tiny_l2")
    E1 = wl.E if dtype == "f32" else workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(wl.E))
    R1 = wl.Rv if dtype == "f32" else workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(wl.Rv))
    delta1 = 0.66 if p == 2 else 2.95
    # second call: fewer entities, fewer relations and a smaller d than the first (ragged: not a multiple of a tile)
    E2, R2 = np.ascontiguousarray(E1[:777, :27]), np.ascontiguousarray(R1[:3, :27])
    delta2 = 0.60 if p == 2 else 2.6
    j = kgc.Join(dtype=dtype, prune=kgc.KGC_PRUNE_OFF)
    try:
        for E, Rv, delta in ((E1, R1, delta1), (E2, R2, delta2)):
            ref = oracle.join(E, Rv, p, delta, mode="abandon")
            assert ref["count"] > 0
            got, st = _both(j, kgc, E, Rv, _dev(E, dtype), _dev(Rv, dtype), p, delta, cap=max(1024, 2 * ref["count"]))
            rep = parity.compare(got, ref, E, Rv, p, delta, E.shape[0])
            assert rep["gpu_count"] == ref["count"] - rep["only_oracle_in_band"] + rep["only_gpu_in_band"]
            assert st["tiles_pruned"] == 0 and st["emitted"] == got["h"].size
    finally:
        j.close()


def test_static_join_runs_in_relation_batches_and_rejects_what_does_not_fit():
    import torch
    import paper_2307_12059_amd as kgc
    # d = 250 -> 8 slices of 64 bytes per row: with N = 40,000 one relation's staged operands take 20 MB, so the 48 MiB
    # array holds the tail operands and ONE relation at a time
    rng = np.random.default_rng(7)
    N, R, d = 40000, 3, 250
    cent = rng.standard_normal((50, d)).astype(np.float32)
    lab = rng.integers(0, 50, N)
    E = (cent[lab] + 0.1 * rng.standard_normal((N, d))).astype(np.float32)
    Rv = (cent[[1, 2, 3]] - cent[[4, 5, 6]]).astype(np.float32)
    delta = 2.05
    j = kgc.Join(dtype="f32", prune=kgc.KGC_PRUNE_OFF)
    try:
        Ed, Rd = _dev(E, "f32"), _dev(Rv, "f32")
        got, st = _both(j, kgc, E, Rv, Ed, Rd, 2, delta, cap=1 << 20)
        assert st["relation_batches"] == R
        hits = got["h"].size
        assert hits > 0
        d64 = oracle.dist_triples(E, Rv, 2, got["h"], got["r"], got["t"])
        assert np.all(d64 <= delta * (1 + 1e-4)) and np.allclose(d64, got["dist"], rtol=1e-4)
        # too large for the array: a clear error, nothing launched, the handle stays usable
        big = torch.zeros((200000, d), dtype=torch.float32, device="cuda")
        out = torch.empty((16, 4), dtype=torch.int32, device="cuda")
        rc, n = kgc.kgc_join_static(j.handle, big.data_ptr(), big.shape[0], d, Rd.data_ptr(), R, 2, 1.0, out.data_ptr(), 16)
        assert rc == kgc.KGC_E_INVALID and n == 0 and "static scratch" in kgc.kgc_last_error(j.handle)
        rc, n = kgc.kgc_join_static(j.handle, Ed.data_ptr(), 300, d, Rd.data_ptr(), R, 2, delta, out.data_ptr(), 16)
        assert rc in (kgc.KGC_OK, kgc.KGC_OVERFLOW)
    finally:
        j.close()
