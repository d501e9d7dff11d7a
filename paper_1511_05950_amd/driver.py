"""Simulated n-softsync training loop on one GPU: sequences the protocol calls of the C library.

Host orchestration only -- every arithmetic step runs in the library's kernels.  lambda learners take
turns round-robin; the l-th gradient of update i comes from learner (i*c + l) mod lambda and is computed on
the weight version i - min(schedule[i][l], i), so the staleness the server sees is the schedule's (clamped
at the start).  This realises the server-view update of the paper's Section 3 for a given staleness trace.
"""
from __future__ import annotations


def run_softsync(ctx, schedule, batch_of, lam, loss_out=None, on_gradient=None, first_update=0):
    """Run len(schedule) server updates.

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
        ctx.sumGradients()
        ctx.applyUpdate()
    return log
