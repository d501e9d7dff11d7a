#!/usr/bin/env python3
"""Writes the stored expected values of the two long bf16 runs (BASELINE configs 3 and 4) from the CPU oracle alone.

    python tests/golden/make_config_runs.py --config 3     # -> tests/golden/config3_run.npz   (about 25 min on 8 cores per mode)
    python tests/golden/make_config_runs.py --config 4     # -> tests/golden/config4_run.npz   (about 5 min per mode, 11 GB of RAM)

Each run is oracle.protocol.run (the server-view iteration of Section 3 with the n-softsync rule of Section 2.2 and
the staleness-dependent rate of Section 2.4) over the config's own seeded images, labels, weights and staleness schedule,
with oracle.cnn as the learners' calcGradient (Section 2.1), once in the exact mode and once in the reduced-precision
mode (tensors between layers rounded to bfloat16).  Nothing here touches the HIP library; the GPU tests load the
files and compare.

config3_run.npz: log [K c][5] = (i, l, learner, j, tau); for both modes the whole update theta_K - theta_0 and the
momentum v after K = 100 updates (float32 copies of the float64 results), and theta_1 - theta_0 of the exact mode
(first_update_exact), which a CPU test recomputes to show that the file belongs to the oracle and inputs as they stand.
config4_run.npz: P = 62 378 344, so the update theta_K - theta_0 after K = 20 updates is stored on a seeded sample: per
weight / bias tensor its first and last 1 024 elements plus 16 384 drawn uniformly (all of it when the tensor is
smaller), with the per-tensor l2 norms of the full update for reference.  A third run of config 4 (update_r32) takes
the reduced-precision mode of the compiled copy of the oracle whose running sums are rounded to float after every term
(make_alex8_bf16_spread.float_sum_copy): one more legitimate bf16 evaluation of the same 20 updates, whose distance to
the reduced-precision run says how far two such evaluations drift apart over the whole run
(`--config 4 --only-r32` adds it to an existing file).
"""
import argparse
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)
sys.path.insert(0, HERE)

import workloads as wl                      # noqa: E402
from oracle import cnn, protocol            # noqa: E402


def tensor_ranges(net):
    out, pos = [], 0
    for ws, nb in wl.param_shapes(net):
        nw = int(np.prod(ws))
        out.append((pos, pos + nw))
        pos += nw
        out.append((pos, pos + nb))
        pos += nb
    return out


def sample_indices(net, seed=4040, edge=1024, draws=16384):
    rng = np.random.default_rng(seed)
    parts = []
    for (a, b) in tensor_ranges(net):
        n = b - a
        if n <= 2 * edge + draws:
            parts.append(np.arange(a, b))
            continue
        mid = rng.choice(n - 2 * edge, size=draws, replace=False) + edge
        parts.append(a + np.concatenate([np.arange(edge), np.sort(mid), np.arange(n - edge, n)]))
    return np.concatenate(parts).astype(np.int64)


def run_mode(cfgd, reduced, progress, K=None, callback=None):
    net, lam, n = cfgd["net"], cfgd["lam"], cfgd["n"]
    X, Y, w0 = cfgd["images"](), cfgd["labels"](), cfgd["weights"]()
    sched = cfgd["schedule"]()
    if K is not None:
        sched = sched[:K]
    R = int(sched.max()) + 1
    t0 = time.time()
    count = [0]

    def watch(i, l, g):
        count[0] += 1
        if count[0] % progress == 0:
            print("  %s: gradient %d (update %d) after %.0f s" % ("reduced" if reduced else "exact", count[0], i, time.time() - t0), flush=True)

    ref = protocol.run(callback or cnn.make_callback(net, round_bf16=reduced), w0,
                       lambda i, l: (X[wl.batch_slice(cfgd, i, l)], Y[wl.batch_slice(cfgd, i, l)]),
                       sched, lam, n, cfgd["alpha0"], cfgd["momentum"], cfgd["weight_decay"], cfgd["lr_mode"], keep=R, on_gradient=watch)
    return ref, w0.astype(np.float64)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, required=True, choices=(3, 4))
    ap.add_argument("--only-r32", action="store_true", help="config 4: add the float-running-sums run to the existing file")
    args = ap.parse_args()
    cfgd = wl.config(args.config)
    net = cfgd["net"]
    out = {}
    path = os.path.join(HERE, "config%d_run.npz" % args.config)
    if args.only_r32:
        out = dict(np.load(path))
    for reduced in (() if args.only_r32 else (False, True)):
        ref, w0 = run_mode(cfgd, reduced, 90 if args.config == 3 else 1)
        tag = "reduced" if reduced else "exact"
        upd = ref["theta"] - w0
        out["log"] = np.asarray(ref["log"], dtype=np.int64)
        if args.config == 3:
            out["update_" + tag] = upd.astype(np.float32)
            out["v_" + tag] = ref["v"].astype(np.float32)
        else:
            idx = sample_indices(net)
            out["idx"] = idx.astype(np.int32)
            out["update_" + tag] = upd[idx].astype(np.float32)
            out["norm_" + tag] = np.array([np.linalg.norm(upd[a:b]) for (a, b) in tensor_ranges(net)])
        del ref
    if args.config == 3:
        ref, w0 = run_mode(cfgd, False, 90, K=1)
        out["first_update_exact"] = (ref["theta"] - w0).astype(np.float32)
    else:
        import tempfile
        import make_alex8_bf16_spread as mk
        with tempfile.TemporaryDirectory() as tmp:
            lg = mk.float_sum_copy(tmp)

            def cb(theta, batch):
                loss, g = lg(net, theta, batch[0], batch[1])
                return g, loss
            ref, w0 = run_mode(cfgd, True, 1, callback=cb)
        out["update_r32"] = (ref["theta"] - w0)[sample_indices(net)].astype(np.float32)
    np.savez_compressed(path, **out)
    print("wrote", path, os.path.getsize(path), "bytes")


if __name__ == "__main__":
    main()
