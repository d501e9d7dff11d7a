"""Event-driven model of where gradient staleness comes from (paper Sections 2.3 and 2.4).

lambda learners loop  pull -> compute -> push  against a parameter server that updates after every
c = floor(lambda / n) pushes.  Pull and push are blocking and instantaneous here; a learner's compute time is
1 + jitter * U(-1, 1) virtual time units (homogeneous processors at similar speed, Section 2.3).  The staleness
of a gradient is the number of server updates between its pull and its push.  Host logic only: the output is
a staleness trace that the driver replays on the GPU (and the oracle on the CPU).

The paper measured (Section 2.4, Figure 1, lambda = 30): 1-softsync gives staleness in {0, 1, 2}; n-softsync
has mean staleness close to n and exceeds 2n with probability below 1e-4.
"""
from __future__ import annotations

import heapq

import numpy as np


def simulate(lam, n, updates, jitter=0.1, seed=0):
    """Return (schedule, learners): int32 [updates][c] staleness of each update's gradients in arrival order
    and the id of the learner that produced each."""
    if not (1 <= n <= lam):
        raise ValueError("n must lie in [1, lambda]")
    c = lam // n
    rng = np.random.default_rng(seed)
    timestamp = 0
    # every learner pulls version 0 at time 0 and finishes its first gradient after its compute time
    heap = [(1.0 + jitter * rng.uniform(-1, 1) + 1e-9 * l, l, 0) for l in range(lam)]   # (finish time, learner, pulled version)
    heapq.heapify(heap)
    schedule = np.zeros((updates, c), np.int32)
    learners = np.zeros((updates, c), np.int32)
    pending = 0
    while timestamp < updates:
        t, l, j = heapq.heappop(heap)
        schedule[timestamp][pending] = timestamp - j          # staleness at push: tau = i - j
        learners[timestamp][pending] = l
        pending += 1
        if pending == c:
            timestamp += 1
            pending = 0
        # the push returns, the learner pulls the current weights and starts its next mini-batch
        heapq.heappush(heap, (t + 1.0 + jitter * rng.uniform(-1, 1), l, timestamp))
    return schedule, learners
