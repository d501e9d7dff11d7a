"""Evaluator of the convergence bound of Section 3 (Theorem 1) for a given staleness trace.

Host-side analysis utility (plain floats, nothing here is on the training path).  Notation of Section 3:
the K updates of c gradients each are unrolled into T = K c one-gradient steps; step t = c i + r uses the
staleness p_t = tau_{i, r} of the r-th gradient of update i.  C1..C4 are the positive constants of the
theorem (properties of the objective), mu the mini-batch size, n the splitting parameter (staleness is at
most 2 n).  A staleness of 0 counts as 1, as in the learning-rate rule.
"""
from __future__ import annotations

import math


def p_sequence(schedule):
    """p_t for t = 0 .. K c - 1 from a staleness table [K][c] (row i = update i, in arrival order)."""
    return [max(int(tau), 1) for row in schedule for tau in row]


def bound_rhs(p, C1, C2, mu):
    """Right-hand side of the theorem's rate: 2 sqrt((2 C1 C2 / mu) sum_t 1/p_t^2) / sum_t 1/p_t."""
    s1 = sum(1.0 / pt for pt in p)
    s2 = sum(1.0 / (pt * pt) for pt in p)
    return 2.0 * math.sqrt(2.0 * C1 * C2 / mu * s2) / s1


def alpha0_star(p, C1, C2, c, mu):
    """The base rate for which the theorem states its bound: sqrt(C1 c^2 mu / sum_t (2 C2 / p_t^2))."""
    s2 = sum(2.0 * C2 / (pt * pt) for pt in p)
    return math.sqrt(C1 * c * c * mu / s2)


def prerequisites_hold(p, alpha0, c, n, C2, C3, C4):
    """The theorem's two conditions on alpha0, checked at every step t.

    (i)  alpha0 <= c C2 / (C3 p_t sum_{j = t-2n}^{t-1} 1/p_j^2)
    (ii) C3 alpha0 / (c p_t) + C4 n alpha0^2 / (c^2 p_t) sum_{k = 1}^{2n} 1/p_{t+k} <= 1
    Window terms that fall outside the trace are left out.  Returns (ok, first_violating_t or None).
    """
    T = len(p)
    for t in range(T):
        back = sum(1.0 / (p[j] * p[j]) for j in range(max(0, t - 2 * n), t))
        if back > 0.0 and alpha0 > c * C2 / (C3 * p[t] * back):
            return False, t
        fwd = sum(1.0 / p[t + k] for k in range(1, 2 * n + 1) if t + k < T)
        if C3 * alpha0 / (c * p[t]) + C4 * n * alpha0 * alpha0 / (c * c * p[t]) * fwd > 1.0:
            return False, t
    return True, None
