"""Deferred updates: consecutive updates whose kernels are launched together, as one pass over theta and v, must leave
exactly the bits that update-by-update launches leave -- weights, momentum and every weight version in the ring."""
import numpy as np
import pytest

import workloads as wl

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def run(net, netarg, compute, lam, mu, n, K, sched, flags, seed, R, alpha0=0.02, momentum=0.9, wd=1e-3, std=0.1):
    from paper_1511_05950_amd import binding, driver
    c = lam // n
    X = wl.images(net, K * c * mu, seed)
    Y = wl.labels(net, K * c * mu, seed + 1)
    w0 = wl.init_weights(net, seed + 2, std=std)
    Xd, Yd = torch.from_numpy(X).cuda(), torch.from_numpy(Y).cuda()
    sl = lambda i, l: slice((i * c + l) * mu, (i * c + l + 1) * mu)
    ctx = binding.Sasgd(lam, mu, n, R, net=netarg, compute=compute, alpha0=alpha0, momentum=momentum, weight_decay=wd, init_weights=w0,
                        flags=flags)
    ctx.setProfiling(True)
    log, calls = driver.run_softsync_batched(ctx, sched, lambda i, l: (Xd[sl(i, l)], Yd[sl(i, l)]), lam)
    _, steps = ctx.phaseTime(1)
    _, passes = ctx.phaseTime(2)
    out = dict(log=log, w=ctx.copyWeights(), v=ctx.copyMomentum(), steps=steps, passes=passes,
               old=[ctx.copyWeights(j) for j in range(max(0, K - R + 1), K)])
    ctx.destroy()
    return out


def same_bits(a, b):
    return np.array_equal(np.asarray(a).view(np.uint32), np.asarray(b).view(np.uint32))


@pytest.mark.parametrize("case", ["fp32_cifar_c1", "bf16_factored_c1", "bf16_factored_c3", "fp32_small_ring"])
def test_fused_steps_leave_the_bits_of_single_updates(case):
    from paper_1511_05950_amd import binding
    fc_net = {"name": "fcnet", "input": (3, 10, 10), "classes": 8,
              "layers": [("conv", 8, 3, 1, 1), ("relu",), ("maxpool", 3, 2), ("fc", 72), ("relu",), ("fc", 24), ("relu",), ("fc", 8)]}
    if case == "fp32_cifar_c1":        # one gradient per update, long bursts: passes of up to 8 steps, ragged last pass
        args = dict(net=wl.CIFAR3, netarg="cifar3", compute="fp32", lam=12, mu=2, n=12, K=45, R=25, std=0.05)
        sched = wl.jitter_schedule(45, 1, 12, 5)
    elif case == "bf16_factored_c1":   # factored fully connected layers between flat stretches, bf16 ring copies
        args = dict(net=fc_net, netarg=fc_net, compute="bf16", lam=10, mu=5, n=10, K=31, R=21)
        sched = wl.jitter_schedule(31, 1, 10, 6)
    elif case == "bf16_factored_c3":   # three gradients per step
        args = dict(net=fc_net, netarg=fc_net, compute="bf16", lam=9, mu=4, n=3, K=14, R=7)
        sched = wl.uniform_schedule(14, 3, 0, 6, 7)
    else:                              # ring shorter than a pass: several steps of one pass take the same slot
        args = dict(net=wl.CIFAR3, netarg="cifar3", compute="fp32", lam=6, mu=2, n=6, K=20, R=3, std=0.05)
        sched = wl.uniform_schedule(20, 1, 1, 2, 8)
    eager = run(sched=sched, flags=binding.FLAG_EAGER_UPDATES, seed=300, **args)
    fused = run(sched=sched, flags=0, seed=300, **args)
    assert eager["log"] == fused["log"]
    assert eager["steps"] == fused["steps"] == len(sched)
    assert eager["passes"] == len(sched) and fused["passes"] < len(sched)       # the default did merge launches
    print(case, "updates", len(sched), "passes", fused["passes"])
    assert same_bits(eager["w"], fused["w"]) and same_bits(eager["v"], fused["v"])
    assert len(eager["old"]) > 0
    for a, b in zip(eager["old"], fused["old"]):
        assert same_bits(a, b)
