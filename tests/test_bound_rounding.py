"""The float32 arithmetic of the L2 tile bound (k_bound_l2 in csrc/kgc_prune.h) against double precision.

The bound test keeps a micro-tile pair under relation r when ||c_H + r - c_T|| <= delta + rho_H + rho_T, evaluated in
float32 from parts that are shared between the tests (Section 4.4's pivot bound with a tile's own centre as the pivot):
    ||c_H + r - c_T||^2 = D[H][T] + 2 (u[r][H] - u[r][T]) + ||r||^2,   D = ||c_H - c_T||^2,  u[r][m] = r . c_m.
For TransE data r nearly cancels c_H - c_T, so D and ||r||^2 are orders of magnitude larger than the reach^2 they are
compared with, and the float32 errors of all of them land on a small difference.  Rounding may only ever KEEP more.
This test re-states the kernel's operation order in numpy float32 and checks, on centres built so that the exact
inequality holds by a hair and D / reach^2 is 10^2 .. 10^5, that the float32 test never drops a pair -- and that it
does drop some once its widening terms are removed (so the check can fail)."""
import numpy as np

F = np.float32
K_BOUND_SLACK = F(2e-4)


def _sum32(x):
    """float32 sum in index order (the order of a plain loop)"""
    s = F(0)
    for v in x.astype(np.float32):
        s = F(s + v)
    return s


def _keeps(cH, cT, r, rH, rT, delta, slack=True):
    d = cH.size
    cH32, cT32, r32 = cH.astype(np.float32), cT.astype(np.float32), r.astype(np.float32)
    D = _sum32((cH32 - cT32) * (cH32 - cT32))
    uH, uT, rn = _sum32(r32 * cH32), _sum32(r32 * cT32), _sum32(r32 * r32)
    ks = K_BOUND_SLACK if slack else F(0)
    cnH = F(np.sqrt(_sum32(cH32 * cH32))) * (F(1) + ks)
    cnT = F(np.sqrt(_sum32(cT32 * cT32))) * (F(1) + ks)
    kk = F(2) * F(d + 12) * F(6e-8) if slack else F(0)
    srn = F(np.sqrt(rn))
    aH = F(F(2) * uH + rn * (F(1) - (F(2.4e-7) if slack else F(0))))
    A2 = F(aH - F(kk * cnH) * srn)
    B2 = F(F(2) * uT + F(kk * cnT) * srn)
    dsl = F(delta) * (F(1) + ks)
    reach = F(F(dsl + F(rH)) + F(rT))
    dk = F(d + 8) * F(6e-8) if slack else F(0)
    rhs = F(F(F(reach * reach) * (F(1) + ks)) + F(D * dk) - D)
    return bool(A2 <= F(rhs + B2))


def test_float32_bound_never_drops_a_pair_that_the_exact_bound_keeps():
    g = np.random.default_rng(77)
    dropped_without_slack = 0
    trials = 0
    for d in (100, 200):
        for scale in (3.0, 10.0, 30.0, 100.0):           # ||r|| ~ scale * sqrt(d) / 10: D / reach^2 from 1e2 to 1e5
            for _ in range(120):
                cH = g.standard_normal(d) * 2.0 + 5.0          # centres far from the origin
                r = g.standard_normal(d) * scale / 10.0
                delta, rH, rT = 0.2, 0.05, 0.05
                reach = delta + rH + rT
                eps = g.standard_normal(d)
                eps *= reach * (1.0 - 1e-9) / np.linalg.norm(eps)     # the exact inequality holds by a hair
                cT = cH + r - eps
                # what the kernel sees are float32 centres: the exact side is taken on those values
                cH64, cT64, r64 = cH.astype(np.float32).astype(np.float64), cT.astype(np.float32).astype(np.float64), r.astype(np.float32).astype(np.float64)
                exact = np.linalg.norm(cH64 + r64 - cT64)
                if exact > reach:                              # rounding the inputs pushed it out: not this test's case
                    continue
                trials += 1
                assert np.sum((cH64 - cT64) ** 2) / reach ** 2 > 50.0
                assert _keeps(cH, cT, r, rH, rT, delta), (d, scale, exact, reach)
                dropped_without_slack += not _keeps(cH, cT, r, rH, rT, delta, slack=False)
    assert trials > 300
    # the check has teeth: with every widening term taken out the float32 test loses pairs
    assert dropped_without_slack > 0
