"""The Theorem 1 evaluator against what Section 3 itself fixes: the constant-staleness remark, the last steps
of the proof (which tie the stated rate to the stated bound), and the remark on concentrated staleness."""
import math

import numpy as np

from paper_1511_05950_amd import theory


def test_constant_staleness_gives_the_one_over_sqrt_mu_T_rate():
    C1, C2, mu = 3.0, 0.7, 16
    for p0 in (1, 4, 30):
        for T in (10, 1000):
            rhs = theory.bound_rhs([p0] * T, C1, C2, mu)
            assert math.isclose(rhs, 2 * math.sqrt(2 * C1 * C2) / math.sqrt(T * mu), rel_tol=1e-12)


def test_stated_rate_turns_the_proofs_bound_into_the_stated_rhs():
    # proof of Theorem 1: (C1 + alpha0^2 sum_t 2 C2 / (mu c^2 p_t^2)) / sum_t alpha0 / (c p_t) equals the
    # stated right-hand side once alpha0 takes the stated value
    rng = np.random.default_rng(1)
    for c, mu in ((1, 4), (3, 16), (18, 128)):
        sched = rng.integers(0, 9, (50, c))
        p = theory.p_sequence(sched)
        assert len(p) == 50 * c and min(p) >= 1
        C1, C2 = 2.5, 0.3
        a = theory.alpha0_star(p, C1, C2, c, mu)
        num = C1 + a * a * sum(2 * C2 / (mu * c * c * pt * pt) for pt in p)
        den = sum(a / (c * pt) for pt in p)
        assert math.isclose(num / den, theory.bound_rhs(p, C1, C2, mu), rel_tol=1e-12)
        # and that rate minimises the proof's expression over alpha0
        for f in (0.5, 0.9, 1.1, 2.0):
            b = f * a
            assert (C1 + b * b * sum(2 * C2 / (mu * c * c * pt * pt) for pt in p)) / sum(b / (c * pt) for pt in p) >= num / den * (1 - 1e-12)


def test_concentrated_staleness_gives_the_smaller_bound():
    # Section 3 remark: with sum_t 1/p_t fixed, the bound is smallest when all p_t are equal
    T = 64
    equal = theory.bound_rhs([4.0] * T, 1.0, 1.0, 1)
    rng = np.random.default_rng(2)
    for _ in range(20):
        z = rng.uniform(0.05, 1.0, T)
        z *= (T / 4.0) / z.sum()                 # same sum of 1/p_t as p_t = 4
        assert theory.bound_rhs(list(1.0 / z), 1.0, 1.0, 1) > equal


def test_prerequisites_hold_for_small_rates_only():
    p = theory.p_sequence(np.random.default_rng(3).integers(1, 9, (40, 2)))
    ok, _ = theory.prerequisites_hold(p, 1e-6, 2, 4, 1.0, 1.0, 1.0)
    assert ok
    bad, t = theory.prerequisites_hold(p, 1e3, 2, 4, 1.0, 1.0, 1.0)
    assert not bad and 0 <= t < len(p)
    # a single step, no history: only condition (ii) applies, C3 alpha0 / (c p) <= 1
    assert theory.prerequisites_hold([2], 3.9, 2, 1, 1.0, 1.0, 1.0)[0]
    assert not theory.prerequisites_hold([2], 4.1, 2, 1, 1.0, 1.0, 1.0)[0]
