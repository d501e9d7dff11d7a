"""Parameter-server iteration of staleness-aware n-softsync ASGD -- TEST INFRASTRUCTURE ONLY.

Follows the paper's notation.  lambda learners, mini-batch mu, splitting parameter n,
c = floor(lambda / n) gradients per update (Section 2.2, n-softsync rule).  The server
keeps a scalar timestamp i, incremented by every update; a gradient carries the
timestamp j of the weights it was computed on, and its staleness is tau = i - j >= 0
(Section 2.1).  Each gradient is scaled by its own learning rate alpha0 / tau
(Section 2.4, staleness-dependent learning rate), the c scaled gradients are averaged
and subtracted from the weights (Section 2.2 n-softsync rule; Section 3, server-view
update equation).

Readings where the paper is silent:
  * tau = 0: the rule of Section 2.4 is stated for tau > 0 only; a fresh gradient gets
    the unmodulated alpha0, i.e. alpha(tau) = alpha0 / max(tau, 1).
  * momentum m and weight decay wd (the paper states "momentum 0.9" without a formula and
    never mentions decay): with coef_l = alpha(tau_l) / c and abar = sum_l coef_l,
        v <- m v + sum_l coef_l g_l + abar wd theta_i ;   theta_{i+1} = theta_i - v .
    At m = wd = 0 this is exactly the n-softsync rule; at lambda = n = 1, tau = 0 it is
    ordinary momentum SGD  v <- m v + alpha0 (g + wd theta).  This convention is shared
    with the GPU path and is otherwise unpinned by the paper.
  * exactly c gradients enter an update, reduced in arrival order l = 0..c-1.
  * a requested staleness larger than the current timestamp is clamped, tau = min(request, i),
    so early gradients read theta_0.
  * learners take turns round-robin: gradient l of update i comes from learner (i c + l) mod lambda.

All arithmetic is float64.
"""
from __future__ import annotations

import numpy as np

PER_GRADIENT = "per_gradient"      # alpha0 / tau_l            (the paper's proposal, Section 2.4)
MEAN_STALENESS = "mean_staleness"  # alpha0 / mean_l(tau_l)    (one rate per update)
CONSTANT = "constant"              # alpha0                    (the paper's comparison arm, Section 4.3 (a))


def softsync_c(lam, n):
    """Gradients per update, c = floor(lambda / n), 1 <= n <= lambda (Section 2.2)."""
    if not (1 <= n <= lam):
        raise ValueError("n must lie in [1, lambda]")
    return lam // n


def learning_rates(taus, alpha0, mode=PER_GRADIENT):
    """alpha_{i,l} for the c gradients of one update (Section 2.4)."""
    taus = np.asarray(taus, dtype=np.int64)
    if (taus < 0).any():
        raise ValueError("staleness is never negative")
    if mode == PER_GRADIENT:
        return alpha0 / np.maximum(taus, 1).astype(np.float64)
    if mode == MEAN_STALENESS:
        return np.full(taus.shape, alpha0 / max(float(taus.mean()), 1.0))
    if mode == CONSTANT:
        return np.full(taus.shape, float(alpha0))
    raise ValueError(mode)


def server_update(theta, v, grads, taus, alpha0, momentum=0.0, weight_decay=0.0, mode=PER_GRADIENT):
    """sumGradients + applyUpdate for one timestamp: returns (theta_next, v_next).

    grads: sequence of c arrays g_l (each the mean gradient of one mini-batch);
    taus: their c staleness values.
    """
    c = len(grads)
    coef = learning_rates(taus, alpha0, mode) / c
    s = np.zeros_like(theta, dtype=np.float64)
    for l in range(c):                       # arrival order
        s += coef[l] * np.asarray(grads[l], dtype=np.float64)
    abar = coef.sum()
    v_next = momentum * v + s + abar * weight_decay * theta
    return theta - v_next, v_next


def step_decay(alpha0, boundaries, factor, K):
    """Base rate of each of K updates when alpha0 is divided by `factor` once update index i has reached each
    boundary (Section 4.3: the rate is lowered by a constant factor after fixed epochs)."""
    out = np.empty(K, np.float64)
    for i in range(K):
        a = float(alpha0)
        for b in boundaries:
            if i >= b:
                a = a / factor
        out[i] = a
    return out


def run(grad_fn, theta0, batches, schedule, lam, n, alpha0, momentum=0.0, weight_decay=0.0,
        mode=PER_GRADIENT, keep=None, on_gradient=None):
    """Run K = len(schedule) server updates.

    alpha0: the base rate, a scalar or an array of K values (one per update, e.g. from step_decay).

    grad_fn(theta, batch) -> (g, loss): a learner's calcGradient on weights theta.
    batches(i, l) -> batch of the l-th gradient of update i.
    schedule: int array [K][c] of requested staleness values.
    keep: if given, weight versions older than i - keep are dropped.
    on_gradient(i, l, g): optional observer.

    Returns dict(theta=final weights, v=momentum, timestamp=K, thetas={version: weights},
                 log=[(i, l, learner, j, tau)], losses=[[loss]*c]*K).
    """
    c = softsync_c(lam, n)
    schedule = np.asarray(schedule)
    K = schedule.shape[0]
    assert schedule.shape == (K, c)
    theta = np.array(theta0, dtype=np.float64)
    v = np.zeros_like(theta)
    thetas = {0: theta.copy()}
    log, losses = [], []
    i = 0                                           # weights timestamp
    for _ in range(K):
        grads, taus, ls = [], [], []
        for l in range(c):
            learner = (i * c + l) % lam
            tau = int(min(int(schedule[i][l]), i))
            j = i - tau                             # timestamp of the pulled weights = of the gradient
            g, loss = grad_fn(thetas[j], batches(i, l))
            if on_gradient is not None:
                on_gradient(i, l, g)
            grads.append(g)
            taus.append(tau)
            ls.append(loss)
            log.append((i, l, learner, j, tau))
        a_i = float(alpha0) if np.ndim(alpha0) == 0 else float(alpha0[i])
        theta, v = server_update(theta, v, grads, taus, a_i, momentum, weight_decay, mode)
        i += 1
        thetas[i] = theta.copy()
        if keep is not None:
            for old in [k for k in thetas if k < i - keep]:
                del thetas[old]
        losses.append(ls)
    return dict(theta=theta, v=v, timestamp=i, thetas=thetas, log=log, losses=losses)


def run_hardsync(grad_fn, theta0, batches, K, lam, alpha, momentum=0.0, weight_decay=0.0):
    """Hardsync / SSGD (Section 2.2, hardsync rule): every update averages lambda gradients
    computed on the current weights (staleness 0) and applies the constant rate alpha."""
    sched = np.zeros((K, lam), dtype=np.int32)
    return run(grad_fn, theta0, batches, sched, lam, 1, alpha, momentum, weight_decay, mode=CONSTANT)
