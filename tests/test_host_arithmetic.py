"""Properties of the arithmetic shortcuts the acceptance kernels take, checked on the CPU in exact rational arithmetic.

Neither test runs device code: each restates a formula the kernels rely on and checks the claim made for it
(the quotient is the correctly rounded one; the interval test never contradicts the exact test)."""
from fractions import Fraction

import numpy as np


def _rn(x: Fraction) -> float:
    return float(x)                    # Fraction -> float is correctly rounded (round to nearest even)


def test_reciprocal_with_one_exact_remainder_gives_the_correctly_rounded_quotient():
    """e / z as q0 = RN(e * RN(1/z)), q = RN(q0 + RN(e - q0 z) * RN(1/z)), the remainder being exact in a fused
    multiply-add: equal to RN(e / z) for every pair drawn from the ranges the kernels see
    (0 < e <= 2.03, an exponential times a table value; 1 <= z < 1e7, a sum of such terms that holds a 1)."""
    rng = np.random.default_rng(7)
    n = 20000
    e = np.exp(-rng.uniform(0.0, 60.0, n)) * rng.uniform(0.99, 2.03, n)
    z = np.concatenate([1.0 + rng.uniform(0.0, 1.0, n // 2) ** 4 * 1e4, rng.uniform(1.0, 1e7, n - n // 2)])
    e[:8] = [2.03, 1.0, 0.5, 1e-30, 1e-200, 3.0 ** -20, 2.0 ** -52, 1.9999999999999998]
    z[:8] = [1.0, 3.0, 1.0000000000000002, 151936.0, 7.0, 49.0, 1e7 - 1.0, 1.9999999999999998]
    for ev, zv in zip(e.tolist(), z.tolist()):
        E, Z = Fraction(ev), Fraction(zv)
        rz = _rn(1 / Z)
        q0 = _rn(E * Fraction(rz))
        rem = _rn(E - Fraction(q0) * Z)                    # what fma(-q0, z, e) returns
        q = _rn(Fraction(q0) + Fraction(rem) * Fraction(rz))
        assert q == _rn(E / Z), (ev, zv)


def test_interval_test_never_contradicts_the_exact_test():
    """The decision takes x < fl32(e / Z) with Z known only as an estimate Zs, |Zs / Z - 1| <= 2^-16: it passes when
    x < fl32(e / (Zs (1 + b))), fails when x >= fl32(e / (Zs (1 - b))), b = 2^-14, and otherwise sums Z exactly.
    Whatever the estimate within its bound, a definite answer must be the exact one."""
    rng = np.random.default_rng(11)
    n = 200000
    b = 2.0 ** -14
    e = np.exp(-rng.uniform(0.0, 30.0, n))
    Z = 1.0 + rng.uniform(0.0, 1.0, n) ** 3 * 2e5
    Zs = Z * (1.0 + rng.uniform(-1.0, 1.0, n) * 2.0 ** -16)
    Zs[::7] = Z[::7] * (1.0 + 2.0 ** -16)                  # the ends of the bound as well
    Zs[1::7] = Z[1::7] * (1.0 - 2.0 ** -16)
    p = (e / Z).astype(np.float32)
    # x close to p, where the interval matters, and far from it
    x = (p.astype(np.float64) * (1.0 + rng.uniform(-1.0, 1.0, n) * rng.choice([1e-7, 1e-5, 1e-4, 1e-3, 0.5], n))).astype(np.float32)
    p_lo = (e / (Zs * (1.0 + b))).astype(np.float32)
    p_hi = (e / (Zs * (1.0 - b))).astype(np.float32)
    definite_pass = x < p_lo
    definite_fail = ~(x < p_hi)
    exact = x < p
    assert not (definite_pass & definite_fail).any()
    assert exact[definite_pass].all()
    assert not exact[definite_fail].any()
    undecided = ~(definite_pass | definite_fail)
    assert 0.2 < undecided.mean() < 0.7                     # most samples were drawn inside or near the band
    far = np.abs(x.astype(np.float64) / np.maximum(p.astype(np.float64), 1e-300) - 1.0) > 2.0e-4
    assert far.any() and not undecided[far & (p > 1e-30)].any()     # and the band is narrow: 2e-4 away is always settled
