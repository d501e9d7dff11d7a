"""GPU parity of the protocol variants around n-softsync: hardsync (Section 2.2), the constant-rate arm
(Section 4.3 (a)), the mean-staleness rate, and replay of a simulated staleness trace (Section 2.4)."""
import numpy as np
import pytest

import workloads as wl
from oracle import cnn, protocol

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def rel(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    return np.linalg.norm(a - b) / np.linalg.norm(b)


def setup(lam, mu, K, c, seed):
    net = wl.CIFAR3
    X = wl.images(net, K * c * mu, seed)
    Y = wl.labels(net, K * c * mu, seed + 1)
    w0 = wl.init_weights(net, seed + 2, std=0.05)
    Xd, Yd = torch.from_numpy(X).cuda(), torch.from_numpy(Y).cuda()
    sl = lambda i, l: slice((i * c + l) * mu, (i * c + l + 1) * mu)
    return net, X, Y, w0, (lambda i, l: (Xd[sl(i, l)], Yd[sl(i, l)])), (lambda i, l: (X[sl(i, l)], Y[sl(i, l)]))


def test_hardsync_matches_oracle_and_big_batch_sgd():
    from paper_1511_05950_amd import binding, driver
    lam, mu, K, alpha = 6, 4, 5, 0.05
    net, X, Y, w0, dev_batch, host_batch = setup(lam, mu, K, lam, 40)
    ctx = binding.Sasgd(lam, mu, 1, 1, net="cifar3", lr_mode="constant", alpha0=alpha, momentum=0.9, init_weights=w0)
    log = driver.run_hardsync(ctx, K, dev_batch, lam)
    w = ctx.copyWeights()
    ctx.destroy()
    ref = protocol.run_hardsync(cnn.make_callback(net), w0, host_batch, K, lam, alpha, momentum=0.9)
    assert log == ref["log"] and all(t == 0 for (_, _, _, _, t) in log)
    assert rel(w - w0, ref["theta"] - w0) < 1e-3
    # hardsync is SGD with mini-batch mu * lambda (Section 2.2): one learner, one big batch, same weights
    Xd, Yd = torch.from_numpy(X).cuda(), torch.from_numpy(Y).cuda()
    one = binding.Sasgd(1, mu * lam, 1, 1, net="cifar3", lr_mode="constant", alpha0=alpha, momentum=0.9, init_weights=w0)
    big = lambda i, l: (Xd[i * lam * mu:(i + 1) * lam * mu], Yd[i * lam * mu:(i + 1) * lam * mu])
    driver.run_softsync(one, [[0]] * K, big, 1)
    w1 = one.copyWeights()
    one.destroy()
    assert rel(w1 - w0, w - w0) < 1e-4


@pytest.mark.parametrize("mode", ["constant", "mean_staleness"])
def test_rate_modes_on_the_network(mode):
    from paper_1511_05950_amd import binding, driver
    lam, mu, n, K = 6, 4, 2, 10
    c = lam // n
    net, X, Y, w0, dev_batch, host_batch = setup(lam, mu, K, c, 50)
    sched = wl.uniform_schedule(K, c, 0, 4, 7)
    ctx = binding.Sasgd(lam, mu, n, 5, net="cifar3", lr_mode=mode, alpha0=0.02, momentum=0.5, weight_decay=1e-3, init_weights=w0)
    log = driver.run_softsync(ctx, sched, dev_batch, lam)
    w = ctx.copyWeights()
    ctx.destroy()
    ref = protocol.run(cnn.make_callback(net), w0, host_batch, sched, lam, n, 0.02, 0.5, 1e-3, mode)
    assert log == ref["log"]
    assert rel(w - w0, ref["theta"] - w0) < 1e-3


def test_simulated_staleness_trace_replay():
    # staleness produced by the event-driven learner/server model instead of a hand-made schedule
    from paper_1511_05950_amd import binding, driver, staleness_sim
    lam, mu, n, K = 12, 4, 12, 80
    sched, _ = staleness_sim.simulate(lam, n, K, jitter=0.2, seed=5)
    assert sched.max() <= 2 * n and abs(sched[20:].mean() - n) < 2
    net, X, Y, w0, dev_batch, host_batch = setup(lam, mu, K, 1, 60)
    ctx = binding.Sasgd(lam, mu, n, int(sched.max()) + 1, net="cifar3", alpha0=0.05, momentum=0.9, init_weights=w0)
    log, calls = driver.run_softsync_batched(ctx, sched, dev_batch, lam)
    w = ctx.copyWeights()
    ctx.destroy()
    ref = protocol.run(cnn.make_callback(net), w0, host_batch, sched, lam, n, 0.05, 0.9)
    assert log == ref["log"]
    assert [t for (_, _, _, _, t) in log] == [int(min(s, i)) for i, s in enumerate(sched[:, 0])]
    assert rel(w - w0, ref["theta"] - w0) < 1e-3


def test_constant_rate_diverges_and_staleness_rate_converges_through_the_server_kernels():
    """The paper's central observation (Section 4.3) through the HIP server path: n-softsync with n = lambda (one
    gradient per update, staleness p) on a linear least-squares model.  With the rate kept at alpha0 the delayed
    iteration is unstable once alpha0 lambda_max exceeds 2 sin(pi / (2 (2p + 1))); with alpha0 / tau (Section 2.4) it
    converges.  The learners' gradients A theta_j - b are formed on the host from the weight version the library holds
    for timestamp j and pushed with that timestamp; pushGradientExternal / sumGradients / applyUpdate do the rest."""
    from paper_1511_05950_amd import binding
    rng = np.random.default_rng(11)
    d, p, K = 48, 15, 600
    Xm = rng.standard_normal((4 * d, d))
    A = Xm.T @ Xm / (4 * d)
    b = rng.standard_normal(d)
    lam_max = np.linalg.eigvalsh(A).max()
    alpha0 = 1.0 / lam_max                                   # stable without delay (limit 2 / lambda_max)
    assert alpha0 * lam_max > 2 * np.sin(np.pi / (2 * (2 * p + 1)))
    star = np.linalg.solve(A, b)
    th0 = rng.standard_normal(d).astype(np.float32)
    e0 = np.linalg.norm(th0 - star)
    sched = np.full((K, 1), p)
    grad_fn = lambda th, batch: (A @ th - b, 0.0)
    out = {}
    for mode in ("constant", "per_gradient"):
        ctx = binding.Sasgd(p, 0, p, p + 1, net=None, num_params=d, lr_mode=mode, alpha0=alpha0, init_weights=th0)
        log = []
        for i in range(K):
            tau = min(p, i)
            th_j = ctx.copyWeights(i - tau).astype(np.float64)
            g = torch.from_numpy((A @ th_j - b).astype(np.float32)).cuda()
            assert ctx.pushGradientExternal(g, i - tau) == tau
            ctx.sumGradients()
            ctx.applyUpdate()
            log.append((i, 0, i % p, i - tau, tau))
            if not np.isfinite(th_j).all():
                break
        w = ctx.copyWeights().astype(np.float64)
        ctx.destroy()
        ref = protocol.run(grad_fn, th0, lambda i, l: None, sched, p, p, alpha0, mode=mode)
        out[mode] = (w, ref, log)
    w, ref, log = out["per_gradient"]
    assert log == ref["log"]
    assert np.linalg.norm(w - star) < 1e-2 * e0 and np.linalg.norm(ref["theta"] - star) < 1e-2 * e0      # converged
    assert rel(w - th0, ref["theta"] - th0) < 1e-4
    w, ref, log = out["constant"]
    assert np.linalg.norm(ref["theta"] - star) > 1e3 * e0                                                 # the oracle diverges
    assert (not np.isfinite(w).all()) or np.linalg.norm(w - star) > 1e3 * e0                              # and so do the kernels
