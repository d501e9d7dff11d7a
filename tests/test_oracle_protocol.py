"""Pins for oracle.protocol: identities and closed forms that fix the n-softsync iteration
(Sections 2.1, 2.2, 2.4 and 3) without reference to the oracle's own code."""
import os

import numpy as np
import pytest

import workloads as wl
from oracle import cnn, protocol

from test_oracle_cnn import gold


def lsq_problem(d=6, m=40, seed=0):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((m, d))
    t = rng.standard_normal(m)
    A = X.T @ X / m
    b = X.T @ t / m
    return A, b


def lsq_callback(A, b):
    return lambda theta, batch: (A @ theta - b, 0.5 * float(theta @ A @ theta) - float(b @ theta))


def test_c_is_floor_lambda_over_n():
    g = gold()
    lam = int(g["softsync_lambda"])
    assert protocol.softsync_c(lam, 15) == g["softsync15_c"]
    assert protocol.softsync_c(lam, 1) == g["softsync1_c"]
    assert protocol.softsync_c(lam, 30) == g["softsync30_c"]
    assert protocol.softsync_c(30, 4) == 7 and protocol.softsync_c(18, 5) == 3
    with pytest.raises(ValueError):
        protocol.softsync_c(4, 5)
    with pytest.raises(ValueError):
        protocol.softsync_c(4, 0)


def test_learning_rate_rule():
    # alpha0 / tau for tau > 0 (Section 2.4); tau = 0 keeps alpha0
    a = protocol.learning_rates([0, 1, 2, 5, 36], 0.01)
    np.testing.assert_allclose(a, [0.01, 0.01, 0.005, 0.002, 0.01 / 36], rtol=1e-15)
    # mean-staleness variant: equal to per-gradient when all tau equal; Jensen gap otherwise
    np.testing.assert_allclose(protocol.learning_rates([3, 3, 3], 0.3, protocol.MEAN_STALENESS),
                               protocol.learning_rates([3, 3, 3], 0.3))
    np.testing.assert_allclose(protocol.learning_rates([1, 3], 0.3, protocol.MEAN_STALENESS), [0.15, 0.15])
    np.testing.assert_allclose(protocol.learning_rates([1, 3], 0.3), [0.3, 0.1])
    np.testing.assert_allclose(protocol.learning_rates([0, 1], 0.3, protocol.MEAN_STALENESS), [0.3, 0.3])
    np.testing.assert_allclose(protocol.learning_rates([4, 9], 0.3, protocol.CONSTANT), [0.3, 0.3])
    with pytest.raises(ValueError):
        protocol.learning_rates([-1], 0.1)


def test_single_learner_is_momentum_sgd():
    # lambda = 1, n = 1: the iteration must be ordinary momentum SGD with weight decay
    A, b = lsq_problem()
    th0 = np.linspace(-1, 1, 6)
    K, a0, m, wd = 25, 0.07, 0.9, 1e-2
    out = protocol.run(lsq_callback(A, b), th0, lambda i, l: None, np.zeros((K, 1), int), 1, 1, a0, m, wd)
    th, v = th0.copy(), np.zeros(6)
    for _ in range(K):
        v = m * v + a0 * ((A @ th - b) + wd * th)
        th = th - v
    np.testing.assert_allclose(out["theta"], th, rtol=1e-12, atol=1e-14)
    assert out["timestamp"] == K
    assert all(t == 0 for (_, _, _, _, t) in out["log"])


def test_zero_staleness_keeps_alpha0_and_equals_hardsync_big_batch():
    # 1-softsync with all tau = 0 == hardsync == one learner with mini-batch mu*lambda (Section 2.2)
    net = wl.tiny_net(2, 8, 8, 3, conv=((3, 3, 1, 1),), pool="avgpool")
    lam, mu, K, a0 = 3, 2, 4, 0.05
    P = wl.num_params(net)
    th0 = np.random.default_rng(3).standard_normal(P) * 0.2
    X = wl.images(net, K * lam * mu, 5).astype(np.float64)
    Y = wl.labels(net, K * lam * mu, 6)
    cb = cnn.make_callback(net)

    def batches(i, l):
        s = (i * lam + l) * mu
        return X[s:s + mu], Y[s:s + mu]
    soft = protocol.run(cb, th0, batches, np.zeros((K, lam), int), lam, 1, a0)
    hard = protocol.run_hardsync(cb, th0, batches, K, lam, a0)
    np.testing.assert_array_equal(soft["theta"], hard["theta"])

    def big(i, l):
        s = i * lam * mu
        return X[s:s + lam * mu], Y[s:s + lam * mu]
    one = protocol.run(cb, th0, big, np.zeros((K, 1), int), 1, 1, a0)
    np.testing.assert_allclose(soft["theta"], one["theta"], rtol=1e-11, atol=1e-14)


def test_plain_sgd_closed_form():
    # no staleness, no momentum: theta_K = theta* + (I - a0 A)^K (theta_0 - theta*)
    A, b = lsq_problem(5, 30, 1)
    th0 = np.ones(5)
    K, a0 = 17, 0.2
    out = protocol.run(lsq_callback(A, b), th0, lambda i, l: None, np.zeros((K, 1), int), 4, 4, a0)
    star = np.linalg.solve(A, b)
    expect = star + np.linalg.matrix_power(np.eye(5) - a0 * A, K) @ (th0 - star)
    np.testing.assert_allclose(out["theta"], expect, rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("p", [1, 2, 5])
def test_delayed_gradient_recurrence_in_eigenbasis(p):
    # c = 1, constant requested staleness p: every eigen-mode of A obeys the scalar delay recurrence
    #   x_{i+1} = x_i - (a0/tau_i) (a x_{i-tau_i} - beta),  tau_i = min(p, i)
    A, b = lsq_problem(6, 50, 2)
    lam = 7
    K, a0 = 40, 0.3
    th0 = np.random.default_rng(4).standard_normal(6)
    out = protocol.run(lsq_callback(A, b), th0, lambda i, l: None, np.full((K, 1), p), lam, lam, a0)
    evals, Q = np.linalg.eigh(A)
    beta = Q.T @ b
    x0 = Q.T @ th0
    final = np.empty(6)
    for k in range(6):
        xs = [x0[k]]
        for i in range(K):
            tau = min(p, i)
            xs.append(xs[i] - (a0 / max(tau, 1)) * (evals[k] * xs[i - tau] - beta[k]))
        final[k] = xs[K]
    np.testing.assert_allclose(out["theta"], Q @ final, rtol=1e-10, atol=1e-12)
    # bookkeeping: timestamps j = i - tau, learners round-robin
    for (i, l, learner, j, tau) in out["log"]:
        assert tau == min(p, i) and j == i - tau and learner == i % lam and l == 0


def test_staleness_counts_updates_not_gradients():
    # Section 3 footnote: three mini-batches computed on the previous weights and pushed into
    # one update all carry staleness 1 in the server-view equation.
    g = gold()
    c = int(g["footnote_minibatches"])
    A, b = lsq_problem()
    sched = np.array([[0] * c, [1] * c])
    out = protocol.run(lsq_callback(A, b), np.zeros(6), lambda i, l: None, sched, c, 1, 0.1)
    second = [tau for (i, l, _, _, tau) in out["log"] if i == 1]
    assert second == [int(g["footnote_staleness"])] * c


def test_one_gradient_per_step_decomposition():
    # Section 3, second update equation: applying the c gradients of an update one at a time, each
    # with rate alpha0 / (c p_t) where p_t is the server-view staleness, lands on the same weights:
    # theta~_{c i} = theta_i.  Gradients are evaluated at the server-view snapshots.
    A, b = lsq_problem(6, 40, 5)
    lam, n, K, a0 = 6, 2, 9, 0.25
    c = lam // n
    sched = wl.uniform_schedule(K, c, 0, 3, 99)
    th0 = np.random.default_rng(8).standard_normal(6)
    out = protocol.run(lsq_callback(A, b), th0, lambda i, l: None, sched, lam, n, a0)
    tilde = th0.copy()
    t = 0
    for i in range(K):
        for r in range(c):
            assert t // c == i and t % c == r
            p_t = min(int(sched[i][r]), i)                    # = tau_{floor(t/c), r_t}
            snapshot = out["thetas"][i - p_t]
            tilde = tilde - a0 / (c * max(p_t, 1)) * (A @ snapshot - b)
            t += 1
        np.testing.assert_allclose(tilde, out["thetas"][i + 1], rtol=1e-12, atol=1e-14)
    # learners take turns: any lambda consecutive gradients come from lambda different learners
    order = [learner for (_, _, learner, _, _) in out["log"]]
    assert all(sorted(order[k:k + lam]) == list(range(lam)) for k in range(len(order) - lam + 1))
    # the footnote's counting: in the decomposed form the staleness of the not-yet-applied
    # gradients grows by one per applied gradient, tau~_t = p_t + r_t
    g = gold()
    assert g["footnote_staleness"] + 1 == g["footnote_decomposed_staleness_next"]


def test_server_update_special_cases_against_numpy():
    rng = np.random.default_rng(0)
    P = 1000
    th = rng.standard_normal(P)
    v = rng.standard_normal(P)
    G = rng.standard_normal((54, P))
    # c = 1, m = wd = 0: an axpy
    t1, v1 = protocol.server_update(th, np.zeros(P), [G[0]], [4], 0.02)
    np.testing.assert_allclose(t1, th - 0.005 * G[0], rtol=1e-14)
    # c = 54, equal tau: scaled column mean
    t2, _ = protocol.server_update(th, np.zeros(P), list(G), [2] * 54, 0.02)
    np.testing.assert_allclose(t2, th - 0.01 * G.mean(axis=0), rtol=1e-12, atol=1e-15)
    # momentum and decay, hand-expanded for c = 2
    t3, v3 = protocol.server_update(th, v, [G[0], G[1]], [0, 3], 0.3, 0.9, 0.01)
    s = 0.15 * G[0] + 0.05 * G[1]
    vv = 0.9 * v + s + 0.2 * 0.01 * th
    np.testing.assert_allclose(v3, vv, rtol=1e-13)
    np.testing.assert_allclose(t3, th - vv, rtol=1e-13)


def test_downpour_is_n_equal_lambda_constant_rate():
    # n = lambda with a constant rate: every single gradient is applied alone with alpha0 (Section 2.2)
    A, b = lsq_problem()
    K, lam, a0 = 12, 5, 0.1
    sched = wl.uniform_schedule(K, 1, 0, 4, 3)
    out = protocol.run(lsq_callback(A, b), np.ones(6), lambda i, l: None, sched, lam, lam, a0,
                       mode=protocol.CONSTANT)
    th = {0: np.ones(6)}
    for i in range(K):
        tau = min(int(sched[i][0]), i)
        th[i + 1] = th[i] - a0 * (A @ th[i - tau] - b)
    np.testing.assert_allclose(out["theta"], th[K], rtol=1e-12)


def test_keep_prunes_old_versions_only():
    A, b = lsq_problem()
    sched = wl.uniform_schedule(20, 2, 0, 3, 1)
    full = protocol.run(lsq_callback(A, b), np.ones(6), lambda i, l: None, sched, 4, 2, 0.1)
    pruned = protocol.run(lsq_callback(A, b), np.ones(6), lambda i, l: None, sched, 4, 2, 0.1, keep=3)
    np.testing.assert_array_equal(full["theta"], pruned["theta"])
    assert min(pruned["thetas"]) == 20 - 3


def test_workload_schedules_have_the_stated_shape():
    # config 2's schedule: mean near n, never above 2n (Section 2.4); config 3's in {0,1,2}
    s2 = wl.config(2)["schedule"]()
    assert s2.shape == (200, 1) and s2.min() >= 0 and s2.max() <= 60 and abs(s2.mean() - 30) < 2
    s3 = wl.config(3)["schedule"]()
    assert s3.shape == (100, 18) and set(np.unique(s3)) == {0, 1, 2}
    s4 = wl.config(4)["schedule"]()
    assert s4.shape == (20, 1) and s4.min() >= 0 and s4.max() <= 36


def test_staleness_dependent_rate_restores_stability():
    # The paper's central observation (Section 4.3): with the rate kept at alpha0, large staleness makes
    # training fail; dividing the rate by the staleness restores it.  On linear least squares with constant
    # delay p the iteration x_{i+1} = x_i - a * lambda_max * x_{i-p} is unstable once a*lambda_max exceeds
    # 2 sin(pi / (2 (2p + 1))) (the classical delayed-gradient bound), far below the undelayed limit of 2.
    A, b = lsq_problem(6, 60, 11)
    lam_max = np.linalg.eigvalsh(A).max()
    p = 15
    alpha0 = 1.0 / lam_max                       # comfortably stable without delay (limit 2 / lam_max)
    assert alpha0 * lam_max > 2 * np.sin(np.pi / (2 * (2 * p + 1)))
    K = 600
    sched = np.full((K, 1), p)
    th0 = np.random.default_rng(1).standard_normal(6)
    star = np.linalg.solve(A, b)
    const = protocol.run(lsq_callback(A, b), th0, lambda i, l: None, sched, p, p, alpha0, mode=protocol.CONSTANT)
    scaled = protocol.run(lsq_callback(A, b), th0, lambda i, l: None, sched, p, p, alpha0)
    e0 = np.linalg.norm(th0 - star)
    assert np.linalg.norm(const["theta"] - star) > 1e3 * e0          # diverged
    assert np.linalg.norm(scaled["theta"] - star) < 1e-2 * e0        # converged
