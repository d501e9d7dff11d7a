"""Simulated n-softsync training loop on one GPU: sequences the protocol calls of the C library.

Host orchestration only -- every arithmetic step runs in the library's kernels.  lambda learners take
turns round-robin; the l-th gradient of update i comes from learner (i*c + l) mod lambda and is computed on
the weight version i - min(schedule[i][l], i), so the staleness the server sees is the schedule's (clamped
at the start).  This realises the server-view update of the paper's Section 3 for a given staleness trace.
"""
from __future__ import annotations


def run_softsync(ctx, schedule, batch_of, lam, loss_out=None, on_gradient=None, first_update=0, base_rates=None):
    """Run len(schedule) server updates.

    base_rates: optional sequence of len(schedule) base learning rates alpha0, one per update (step decay of
    Section 4.3); set with setBaseRate before each update's window is closed.

    ctx: binding.Sasgd;  schedule: int [K][c] requested staleness;  batch_of(i, l) -> (images_dev, labels_dev).
    loss_out: optional device float tensor [c] receiving each update's per-gradient mean losses.
    on_gradient(i, l, learner): optional hook called after calcGradient (e.g. to copy gradients out).
    Returns the log [(i, l, learner, j, tau)] with j the gradient's timestamp and tau its staleness as
    reported by the library.
    """
    c = ctx.c
    log = []
    for k in range(len(schedule)):
        i = first_update + k
        assert ctx.timestamp() == i
        learners = []
        stamps = []
        for l in range(c):
            learner = (i * c + l) % lam
            x, y = batch_of(i, l)
            ctx.getMinibatch(learner, x, y)
            stamps.append(ctx.pullWeights(learner, int(schedule[k][l])))
            learners.append(learner)
        ctx.calcGradient(learners, loss_out)
        for l in range(c):
            if on_gradient is not None:
                on_gradient(i, l, learners[l])
            tau = ctx.pushGradient(learners[l])
            log.append((i, l, learners[l], stamps[l], tau))
        if base_rates is not None:
            ctx.setBaseRate(float(base_rates[k]))
        ctx.sumGradients()
        ctx.applyUpdate()
    ctx.flush()                                 # nothing of this run is left waiting for a later call
    return log


def run_softsync_batched(ctx, schedule, batch_of, lam, loss_out=None, first_update=0):
    """Same run as run_softsync with calcGradient calls merged across updates.

    The lambda learners of the paper work concurrently; a learner whose weights (version j) already exist can
    compute before the update that will consume its gradient.  Whenever an update's gradients are not all
    available, every gradient of the next lambda (one per learner) whose pulled version already exists is
    computed in the same batched call.  Versions, timestamps and staleness are those of run_softsync; only the
    grouping of kernel launches changes.  The ring must hold max(schedule) + 1 versions.
    """
    c = ctx.c
    K = len(schedule)
    done = {}                                   # gradient id -> (learner, timestamp j)
    log = []
    calls = 0
    for k in range(K):
        i = first_update + k
        assert ctx.timestamp() == i
        if any((k * c + l) not in done for l in range(c)):
            learners = []
            for g in range(k * c, min(K * c, k * c + lam)):
                if g in done:
                    continue
                k2, l2 = divmod(g, c)
                i2 = first_update + k2
                j = i2 - min(int(schedule[k2][l2]), i2)
                if j > i:
                    continue                    # its weights do not exist yet
                learner = (i2 * c + l2) % lam
                x, y = batch_of(i2, l2)
                ctx.getMinibatch(learner, x, y)
                got = ctx.pullWeights(learner, i - j)
                assert got == j
                done[g] = (learner, j)
                learners.append(learner)
            ctx.calcGradient(learners, loss_out if len(learners) == c else None)
            calls += 1
        for l in range(c):
            learner, j = done.pop(k * c + l)
            tau = ctx.pushGradient(learner)
            log.append((i, l, learner, j, tau))
        ctx.sumGradients()
        ctx.applyUpdate()
    ctx.flush()
    return log, calls


def run_hardsync(ctx, K, batch_of, lam, loss_out=None):
    """Hardsync / SSGD (paper Section 2.2, hardsync rule): every update averages the gradients of all lambda
    learners computed on the current weights (staleness 0) and applies the constant rate.

    The context must have been created with n = 1 (so c = lambda) and lr_mode "constant".  Returns the log of
    run_softsync (every staleness is 0)."""
    if ctx.c != lam:
        raise ValueError("hardsync needs n = 1 (c = lambda)")
    return run_softsync(ctx, [[0] * lam for _ in range(K)], batch_of, lam, loss_out)


def evaluate(ctx, images_dev, labels_dev, lam, mu, loss_dev, rank_dev, staleness=0):
    """Evaluation pass (test / validation error of Section 4.3) over len(images_dev) = B * mu images on the weight
    version `staleness` updates old: forward only, in batched calls of up to lambda mini-batches.

    loss_dev: device float tensor [B] (mean loss per mini-batch); rank_dev: device int32 tensor [B * mu] (rank of
    the true class; >= 1 is a top-1 error, >= 5 a top-5 error).  Host sequencing only."""
    total = int(images_dev.shape[0])
    if total % mu:
        raise ValueError("the evaluation set must be a whole number of mini-batches")
    B = total // mu
    for b0 in range(0, B, lam):
        nb = min(lam, B - b0)
        for k in range(nb):
            s0 = (b0 + k) * mu
            ctx.getMinibatch(k, images_dev[s0:s0 + mu], labels_dev[s0:s0 + mu])
            ctx.pullWeights(k, staleness)
        ctx.evaluate(list(range(nb)), loss_dev[b0:b0 + nb], rank_dev[b0 * mu:(b0 + nb) * mu])
