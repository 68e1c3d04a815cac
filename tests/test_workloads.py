"""Host-side checks of the seeded input generator (no join arithmetic lives there)."""
import numpy as np
import pytest

import workloads


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.005859375, 1.01171875, -2.5, 3.0e38, 1e-40, 0.0], np.float32)
    b = workloads.f32_to_bf16_bits(x)
    y = workloads.bf16_bits_to_f32(b)
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> even mantissa (1.0); 1 + 3*2^-9 -> 1 + 2^-7;
    # 1 + 3*2^-8 is a tie between 1 + 2^-7 (odd) and 1 + 2^-6 (even) -> 1 + 2^-6
    assert y[0] == 1.0 and y[1] == 1.0 and y[2] == 1.0078125 and y[3] == 1.015625 and y[4] == -2.5
    assert np.all(np.abs(y[:5] - x[:5]) <= np.abs(x[:5]) * 2.0 ** -8)
    assert workloads.f32_to_bf16_bits(y).tolist() == b.tolist()          # idempotent


def test_generator_is_deterministic_and_shaped():
    a = workloads.generate("c1_tiny_l2"); b = workloads.generate("c1_tiny_l2")
    assert a.E.shape == (2000, 32) and a.Rv.shape == (8, 32) and a.E.dtype == np.float32
    assert np.array_equal(a.E, b.E) and np.array_equal(a.Rv, b.Rv) and a.delta == b.delta
    assert a.delta is not None and a.delta == float(np.float32(a.delta))
    assert np.all(a.rel_src != a.rel_dst)
    # within-cluster spread and centre scale are the stated ones
    c0 = a.E[a.labels == a.labels[0]]
    assert abs(c0.std(0).mean() - 0.1) < 0.02 and 0.7 < a.E.std() < 1.3


def test_bf16_storage_values_are_representable():
    wl = workloads.generate("c4_large_l2", N=500, R=4, K=10)
    assert wl.E_bits.dtype == np.uint16 and wl.delta is None
    assert np.array_equal(workloads.bf16_bits_to_f32(wl.E_bits), wl.E)
    assert np.array_equal(workloads.f32_to_bf16_bits(wl.E), wl.E_bits)


def test_zipf_sizes():
    wl = workloads.generate("c5_scale_l2", N=20000, R=5, K=100)
    sizes = np.sort(np.bincount(wl.labels, minlength=100))[::-1]
    assert sizes.sum() == 20000 and sizes.min() >= 1 and sizes[0] > 10 * sizes[50]


def test_samplers():
    wl = workloads.generate("c2_mid_l2", N=3000, R=20, K=50)
    h, r, t = workloads.sample_aligned_triples(wl, 1000, 3)
    assert np.all(wl.labels[h] == wl.rel_src[r]) and np.all(wl.labels[t] == wl.rel_dst[r])
    ent, rel = workloads.cluster_aligned_subsample(wl, 3, 10_000, 5)
    assert set(wl.labels[ent]) == set(wl.rel_src[rel]) | set(wl.rel_dst[rel])
    assert workloads.aligned_triple_count(wl) == sum(
        int((wl.labels == i).sum()) * int((wl.labels == j).sum()) for i, j in zip(wl.rel_src, wl.rel_dst))


@pytest.mark.parametrize("name", list(workloads.SPECS))
def test_stored_deltas_exist(name):
    assert workloads.stored_delta(name) is not None and workloads.stored_delta(name) > 0
