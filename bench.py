#!/usr/bin/env python3
"""Benchmark of the staleness-aware n-softsync ASGD hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload all|alex|server|cifar|cifar-fp32-c4|cifar-fp32-c1|alex-calc|alex-calc-shared|cifar-calc]

Default workload "all": the whole metric in one line.  The line itself is BASELINE config 4 end to end in steady state
(AlexNet-shaped net, bf16 compute with fp32 master weights, lambda = 18 learners of mu = 16, 18-softsync, seeded
staleness uniform in 0..36): one step = one server update = one learner's calcGradient (batched with the other learners
whose weight version already exists) + sumGradients + applyUpdate; value = training images/s; roofline = the
calcGradient launches against the bf16 MFMA peak; roofline_hbm = applyUpdate as it runs inside that step against the HBM
peak.  The ring is pre-warmed by 36 untimed updates whatever --warmup says, so that requested staleness is never
clamped (the literal run from theta_0, where most early gradients read version 0, is the nested "cold_start").  Nested
under further keys: "calc_only" (one batched calcGradient call of all 18 learners, a weight version each),
"server_config1" (BASELINE config 1, P = 60 M fp32, 54 gradients resident: 54 updates at c = 1 and one at c = 54).
"--workload server" prints config 1 as the line itself: one step consumes every learner's gradient once in each of the two
protocols (54-softsync: 54 updates of 20 B per parameter; 1-softsync: one update of 232 B per parameter) and the value is
algorithmic HBM bytes (4 (c + 4) per parameter and update) over wall time.  "cifar", "cifar-fp32-c4", "cifar-fp32-c1"
run the whole path on BASELINE configs 3, 0, 2; "alex-calc" / "cifar-calc" time calcGradient alone with all lambda
learners in one batched call (alex-calc: every learner on a weight version of its own, as under lambda-softsync;
alex-calc-shared: all on one version).
Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# HBM bytes per launch of the update kernel at P = 60e6.  NOT measured by this run: taken from rocprofv3 --pmc
# FETCH_SIZE / WRITE_SIZE runs of this script scaled by a plain 240 MB copy in the same run (summary:
# profiles/apply_update_config1.txt); the line says so in "traffic_source".
TRAFFIC_C1 = 1.2000e9
TRAFFIC_C54 = 14.402e9      # the two-pass form writes and re-reads its sums: + 2 x 240 MB
TRAFFIC_SOURCE = "rocprofv3 --pmc FETCH_SIZE/WRITE_SIZE, profiles/apply_update_config1.txt (not measured by this run)"
# Counted / algorithmic HBM bytes of an update pass of BASELINE config 4 (fused steps, factored fully connected layers),
# from the same two counters over `--workload alex` (summary: profiles/apply_update_config4_fused.txt).
TRAFFIC_RATIO_CFG4 = 1.011
TRAFFIC_SOURCE_CFG4 = ("bytes_per_launch x 1.011 = counted / algorithmic bytes of rocprofv3 --pmc FETCH_SIZE/WRITE_SIZE runs, "
                       "profiles/apply_update_config4_fused.txt (not measured by this run)")
PREWARM_CFG4 = 36           # updates that fill the ring of BASELINE config 4 before anything is timed


def cpu_baseline_server(cfg, budget_s=12.0):
    """The oracle's server update, as it stands, on a slice of the same workload."""
    import numpy as np
    from oracle import protocol
    Ps = 1 << 21
    lam = cfg["lam"]
    rng = np.random.default_rng(0)
    th = rng.standard_normal(Ps) * 0.01
    v = np.zeros(Ps)
    G = [rng.standard_normal(Ps) * 1e-3 for _ in range(lam)]
    taus = cfg["staleness"]()
    t0 = time.perf_counter()
    nbytes = 0
    reps = 0
    while time.perf_counter() - t0 < budget_s:
        for l in range(lam):                                   # 54-softsync: c = 1
            th, v = protocol.server_update(th, v, [G[l]], [int(taus[l])], cfg["alpha0"], cfg["momentum"], cfg["weight_decay"])
        th, v = protocol.server_update(th, v, G, [int(t) for t in taus], cfg["alpha0"], cfg["momentum"], cfg["weight_decay"])
        nbytes += Ps * (lam * 20 + 4 * (lam + 4))
        reps += 1
    dt = time.perf_counter() - t0
    return {"value": nbytes / dt / 1e9, "unit": "GB/s", "cores": 1, "host_cores": os.cpu_count(), "kind": "oracle",
            "sample": "%d steps of the same two protocols on a %d-element slice of the parameter vector "
                      "(numpy fp64 oracle; bytes counted with the fp32 formula 4(c+4) per parameter)" % (reps, Ps)}


def bench_server(args):
    import numpy as np
    import torch
    import workloads as wl
    from paper_1511_05950_amd import binding

    cfg = wl.config(1)
    P, lam = cfg["num_params"], cfg["lam"]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(wl.SEED0 + 1000)
    theta0 = torch.randn(P, device=dev, generator=gen) * 0.01
    grads = [torch.randn(P, device=dev, generator=gen) * 1e-3 for _ in range(lam)]
    taus = cfg["staleness"]()
    kw = dict(net=None, num_params=P, alpha0=cfg["alpha0"], momentum=cfg["momentum"], weight_decay=cfg["weight_decay"])
    ctxA = binding.Sasgd(lam, 0, 54, 1, init_weights=theta0, **kw)     # 54-softsync, c = 1
    ctxB = binding.Sasgd(lam, 0, 1, 1, init_weights=theta0, **kw)      # 1-softsync,  c = 54

    def step():
        i = ctxA.timestamp()
        for l in range(lam):
            ctxA.pushGradientExternal(grads[l], i + l - min(int(taus[l]), i + l))
            ctxA.sumGradients()
            ctxA.applyUpdate()
        j = ctxB.timestamp()
        for l in range(lam):
            ctxB.pushGradientExternal(grads[l], j - min(int(taus[l]), j))
        ctxB.sumGradients()
        ctxB.applyUpdate()

    if args.calibrate_copy:
        # a plain device-to-device copy of one gradient (240 MB read + 240 MB written): the reference the
        # rocprofv3 FETCH_SIZE / WRITE_SIZE counters of the update kernels are scaled by
        scratch = torch.empty_like(grads[0])
        for l in range(3):
            scratch.copy_(grads[l])
        torch.cuda.synchronize()
        del scratch
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ctxA.setProfiling(True)
    ctxB.setProfiling(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    msA, nA = ctxA.phaseTime(1)
    msB, nB = ctxB.phaseTime(1)
    ctxA.destroy()
    ctxB.destroy()

    bytes_step = P * (lam * 20 + 4 * (lam + 4))
    value = bytes_step * args.steps / dt / 1e9
    kA = msA / nA * 1e-3                      # average duration of one c=1 launch, seconds
    kB = msB / nB * 1e-3
    achA = P * 20 / kA / 1e9
    achB = P * 4 * (lam + 4) / kB / 1e9
    out = {
        "metric": "applyUpdate HBM GB/s", "value": round(value, 1), "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(dt / args.steps * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "BASELINE config 1: server update microbench, P=60e6 fp32, lambda=54; one step = "
                               "54 updates at c=1 (54-softsync) + 1 update at c=54 (1-softsync)",
                   "num_params": P, "lambda": lam, "momentum": cfg["momentum"], "weight_decay": cfg["weight_decay"]},
        "roofline": {"bound": "hbm", "kernel": "apply_update_kernel (c=1)", "achieved": round(achA, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achA / HBM_PEAK_GBS, 4), "traffic": TRAFFIC_C1,
                     "traffic_source": TRAFFIC_SOURCE, "avg_launch_us": round(kA * 1e6, 2), "bytes_per_launch": P * 20},
        "roofline_c54": {"bound": "hbm", "kernel": "sum_gradients_kernel + apply_update_kernel per stretch of 2 Mi parameters (c=54, 58 launches)", "achieved": round(achB, 1),
                         "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achB / HBM_PEAK_GBS, 4), "traffic": TRAFFIC_C54,
                         "traffic_source": TRAFFIC_SOURCE, "avg_launch_us": round(kB * 1e6, 2), "bytes_per_launch": P * 4 * (lam + 4)},
    }
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline_server(cfg)
    return out


def cpu_baseline_net(cfg, budget_s=10.0):
    """The oracle's calcGradient, as it stands, on mini-batches of the same workload."""
    import numpy as np
    import workloads as wl
    from oracle import cnn
    net, mu = cfg["net"], cfg["mu"]
    w0 = cfg["weights"]()
    X = wl.images(net, mu, 123)
    Y = wl.labels(net, mu, 124)
    cnn.loss_and_gradient(net, w0, X[:1], Y[:1])                 # builds / loads the library
    t0 = time.perf_counter()
    n = 0
    while time.perf_counter() - t0 < budget_s:
        cnn.loss_and_gradient(net, w0, X, Y)
        n += 1
    dt = time.perf_counter() - t0
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": n * mu / dt, "unit": "images/s", "cores": cores, "host_cores": os.cpu_count(), "kind": "oracle",
            "sample": "%d calcGradient calls of one mini-batch (mu = %d) by the fp64 C oracle with OpenMP; the server update "
                      "is not included" % (n, mu)}


def activation_bytes_per_image(net, elem):
    """Bytes of activations a layer-by-layer (unfused) forward + backward pass has to move per image: forward every layer
    reads its input and writes its output; backward it reads its output gradient and its input (weight gradient, masks
    and pooling winners) and writes its input gradient.  elem = bytes per stored activation; the input image is fp32."""
    c, h, w = net["input"]
    total = c * h * w * 4
    for L in net["layers"]:
        i_el = c * h * w
        if L[0] == "conv":
            _, co, k, st, pd = L
            h = (h + 2 * pd - k) // st + 1
            w = (w + 2 * pd - k) // st + 1
            c = co
        elif L[0] in ("maxpool", "avgpool"):
            _, k, st = L
            ho = -(-(h - k) // st) + 1
            wo = -(-(w - k) // st) + 1
            h = ho - 1 if (ho - 1) * st >= h else ho
            w = wo - 1 if (wo - 1) * st >= w else wo
        elif L[0] == "fc":
            c, h, w = L[1], 1, 1
        elif L[0] == "relu":
            continue                      # fused into the layer in front of it
        o_el = c * h * w
        total += (i_el + o_el) * elem     # forward
        total += (2 * o_el + 2 * i_el) * elem   # backward
    return total


def bench_net(args, cfg_id, prewarm=0, cold=False):
    """Whole hot path on BASELINE config 3 (CIFAR-shaped, bf16, 1-softsync) or 4 (AlexNet-shaped, bf16, 18-softsync):
    one step = one server update = c calcGradients (batched launches) + sumGradients + applyUpdate.
    prewarm: untimed updates in front of the --warmup ones (fills the ring so that no requested staleness is clamped).
    cold: the literal run from theta_0 -- no warm-up update at all, the config's own K updates are the timed steps (one
    identical untimed run on another context first, so that code objects are loaded)."""
    import numpy as np
    import torch
    import workloads as wl
    from paper_1511_05950_amd import binding, driver

    cfg = wl.config(cfg_id)
    net, lam, mu, n, c = cfg["net"], cfg["lam"], cfg["mu"], cfg["n"], cfg["c"]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    warm = 0 if cold else prewarm + args.warmup
    steps = cfg["K"] if cold else args.steps
    K = warm + steps
    rng = np.random.default_rng(wl.SEED0 + 1000 * cfg_id + 3)
    hi = {0: 4, 2: 60, 3: 2, 4: 36}[cfg_id]
    if cfg_id == 2:
        sched = wl.jitter_schedule(K, c, n, wl.SEED0 + 2003)
    else:
        sched = rng.integers(0, hi + 1, size=(K, c)).astype(np.int32)
    if cold:
        sched = cfg["schedule"]()              # the config's own schedule, update for update
    R = hi + 1
    pool = min(cfg["n_images"], 4096)
    pool -= pool % mu
    X = torch.randn((pool,) + net["input"], device=dev, generator=torch.Generator(device=dev).manual_seed(cfg_id))
    Y = torch.randint(0, net["classes"], (pool,), device=dev, dtype=torch.int32)
    w_init = cfg["weights"]()

    def make_ctx():
        return binding.Sasgd(lam, mu, n, R, net=net["name"], compute=cfg["compute"], alpha0=cfg["alpha0"], momentum=cfg["momentum"],
                             weight_decay=cfg["weight_decay"], init_weights=w_init)

    def batch_of(i, l):
        s0 = ((i * c + l) * mu) % pool
        return X[s0:s0 + mu], Y[s0:s0 + mu]

    if cold:
        tmp = make_ctx()
        driver.run_softsync_batched(tmp, sched, batch_of, lam)
        torch.cuda.synchronize()
        tmp.destroy()
    if args.calibrate_copy:
        # plain device-to-device copies of known size (240 MB read + 240 MB written): the reference the rocprofv3
        # FETCH_SIZE / WRITE_SIZE counters of the update kernels are scaled by
        src = torch.zeros(60_000_000, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    ctx = make_ctx()
    # learners whose weights already exist are computed in one batched call (same versions, same staleness)
    driver.run_softsync_batched(ctx, sched[:warm], batch_of, lam)
    torch.cuda.synchronize()
    # the timed steps, as a caller runs them ...
    t0 = time.perf_counter()
    _, calls = driver.run_softsync_batched(ctx, sched[warm:warm + steps], batch_of, lam, first_update=warm)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # ... and the same steps again on a second context brought to the same point, with the phase timer on (HIP events
    # around each phase on the library's stream) for the roofline figures
    ctx.destroy()
    ctx = make_ctx()
    driver.run_softsync_batched(ctx, sched[:warm], batch_of, lam)
    torch.cuda.synchronize()
    ctx.setProfiling(True)
    driver.run_softsync_batched(ctx, sched[warm:], batch_of, lam, first_update=warm)
    torch.cuda.synchronize()
    ms_g, n_g = ctx.phaseTime(0)
    ms_u, n_u = ctx.phaseTime(1)
    _, n_pass = ctx.phaseTime(2)   # passes over the vector: consecutive updates are applied in one pass (fused steps)
    P = ctx.P
    Wf = ctx.factoredParams()      # fully connected weights whose gradient is formed inside applyUpdate from its factors
    ctx.destroy()
    images = steps * c * mu
    flop_img = {0: 68.87424e6, 2: 68.87424e6, 3: 68.87424e6, 4: 6.585512448e9}[cfg_id]   # forward + backward MACs x 2 per image
    flop_img -= 2.0 * Wf           # those weight-gradient MACs are not done by calcGradient
    fp32 = cfg["compute"] == "fp32"
    peak = 157.3 if fp32 else 2500.0
    t_grad = ms_g * 1e-3                                      # all calcGradient calls of the timed region, seconds
    ach = images * flop_img / t_grad / 1e12
    # algorithmic bytes of one update: theta, v read and written, a 2-byte copy in bf16 compute, and 4 bytes per pending
    # gradient for every parameter whose gradient is a written-out vector
    upd_bytes = P * (16 + (0 if fp32 else 2)) + (P - Wf) * 4 * c
    # algorithmic bytes of one pass that applies k updates: theta and v read once, v written once (fp32 master weights
    # too in bf16 compute), and per update its weight version (fp32 ring slot or bf16 copy) and its gradients
    k_pass = n_u / max(n_pass, 1)
    pass_bytes = P * (12 + (0 if fp32 else 4)) + k_pass * (P * (4 if fp32 else 2) + (P - Wf) * 4 * c)
    how = ("cold start: the config's %d updates from theta_0, no warm-up update" % steps if cold else
           "steady state: %d + %d untimed updates first" % (prewarm, args.warmup) if prewarm else "%d untimed updates first" % args.warmup)
    upd_us = ms_u / n_u * 1e3
    pass_us = ms_u / max(n_pass, 1) * 1e3
    out = {
        "metric": "training images/sec per GPU", "value": round(images / dt, 1), "unit": "images/s", "n_gpus": 1,
        "steps": steps, "warmup": warm, "ms_per_step": round(dt / steps * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32" if fp32 else "bf16", "data": "synthetic",
        "config": {"workload": "BASELINE config %d: %s net, lambda=%d, mu=%d, %d-softsync (c=%d), %s; %s"
                               % (cfg_id, net["name"], lam, mu, n, c, "fp32 compute" if fp32 else "bf16 compute, fp32 master", how),
                   "num_params": P, "ring_depth": R, "calcGradient_calls": n_g},
        "roofline": {"bound": "alu" if fp32 else "mfma", "kernel": "calcGradient phase (every launch of its %d batched calls; algorithmic "
                                                "flop = 2 x forward+backward MACs of %d images)" % (n_g, images),
                     "achieved": round(ach, 2), "peak": peak, "unit": "TFLOP/s", "frac": round(ach / peak, 5),
                     "traffic": None, "avg_call_us": round(t_grad / n_g * 1e6, 1), "learners_per_call": round(images / mu / n_g, 2)},
        "roofline_hbm": {"bound": "hbm", "kernel": "applyUpdate as it runs inside the step: one pass over theta and v applies the updates that "
                                                   "are ready together (%.2f per pass on average); bytes = theta, v read and v%s written once per "
                                                   "pass + per update its weight version and its gradients" % (k_pass, "" if fp32 else ", theta"),
                         "achieved": round(pass_bytes / (pass_us * 1e-6) / 1e9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": round(pass_bytes / (pass_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                         "traffic": int(pass_bytes * TRAFFIC_RATIO_CFG4) if cfg_id == 4 else None,
                         "traffic_source": TRAFFIC_SOURCE_CFG4 if cfg_id == 4 else None,
                         "avg_launch_us": round(pass_us, 2), "bytes_per_launch": int(pass_bytes), "updates_per_pass": round(k_pass, 3),
                         "per_update_us": round(upd_us, 2), "lone_update_bytes": upd_bytes,
                         "lone_update_equivalent_GBs": round(upd_bytes / (upd_us * 1e-6) / 1e9, 1), "factored_fc_weights": Wf},
        "phase_ms_per_step": {"calcGradient": round(ms_g / steps, 4), "applyUpdate": round(ms_u / steps, 4)},
    }
    if cfg_id == 3:
        # the small-channel CIFAR-shaped layers are bound by moving activations, not by the matrix cores: report the
        # calcGradient phase against the HBM peak as well (bytes of a layer-by-layer pass, see activation_bytes_per_image)
        act = activation_bytes_per_image(net, 2) * images
        out["roofline_activations"] = {"bound": "hbm", "kernel": "calcGradient phase, activation traffic of a layer-by-layer pass",
                                       "achieved": round(act / t_grad / 1e9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                       "frac": round(act / t_grad / 1e9 / HBM_PEAK_GBS, 4), "traffic": None,
                                       "bytes_per_image": activation_bytes_per_image(net, 2)}
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline_net(cfg)
    return out


def bench_calc(args, cfg_id, shared=False):
    """calcGradient alone (the learners' half of the path): all lambda learners of BASELINE config 3 or 4 in ONE
    batched call per step; no server update inside the timed region."""
    import torch
    import workloads as wl
    from paper_1511_05950_amd import binding

    cfg = wl.config(cfg_id)
    net, lam, mu = cfg["net"], cfg["lam"], cfg["mu"]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    X = torch.randn((lam * mu,) + net["input"], device=dev, generator=torch.Generator(device=dev).manual_seed(cfg_id))
    Y = torch.randint(0, net["classes"], (lam * mu,), device=dev, dtype=torch.int32)
    # 1-softsync (config 3): every learner pulls the version the last update made.  lambda-softsync (config 4): each
    # learner holds a weight version of its own, as it does when gradients are applied one at a time; the versions
    # are made here by lambda updates with a zero gradient (weight decay alone moves them).
    distinct = cfg["n"] > 1 and not shared
    ctx = binding.Sasgd(lam, mu, lam, lam + 1 if distinct else 1, net=net["name"], compute=cfg["compute"], init_weights=cfg["weights"](),
                        alpha0=cfg["alpha0"], momentum=cfg["momentum"], weight_decay=cfg["weight_decay"])
    learners = list(range(lam))
    if distinct:
        zero = torch.zeros(ctx.P, device=dev)
        for _ in range(lam):
            ctx.pushGradientExternal(zero, ctx.timestamp())
            ctx.sumGradients()
            ctx.applyUpdate()
        del zero

    def step():
        for L in learners:
            ctx.getMinibatch(L, X[L * mu:(L + 1) * mu], Y[L * mu:(L + 1) * mu])
            ctx.pullWeights(L, L if distinct else 0)
        ctx.calcGradient(learners)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ctx.setProfiling(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_g, n_g = ctx.phaseTime(0)
    P = ctx.P
    Wf = ctx.factoredParams()
    ctx.destroy()
    images = args.steps * lam * mu
    flop_img = {3: 68.87424e6, 4: 6.585512448e9}[cfg_id] - 2.0 * Wf   # factored fc weight gradients are formed by applyUpdate
    ach = images * flop_img / (ms_g * 1e-3) / 1e12
    out = {
        "metric": "calcGradient images/sec per GPU (no server update)", "value": round(images / dt, 1), "unit": "images/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(dt / args.steps * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "calcGradient only, shapes of BASELINE config %d: %s net, %d learners x mu=%d in one batched call, "
                               "bf16 compute, %s" % (cfg_id, net["name"], lam, mu,
                                                     "one weight version per learner" if distinct else "all learners on one weight version"),
                   "num_params": P},
        "roofline": {"bound": "mfma", "kernel": "calcGradient (all launches of one batched call of %d learners)" % lam,
                     "achieved": round(ach, 2), "peak": 2500.0, "unit": "TFLOP/s", "frac": round(ach / 2500.0, 5),
                     "traffic": None, "avg_call_us": round(ms_g / n_g * 1e3, 1), "learners_per_call": lam},
    }
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline_net(cfg)
    return out


def bench_all(args):
    """The default line: BASELINE config 4 end to end in steady state, with the other parts of the metric nested."""
    import copy
    import gc
    import torch
    out = bench_net(args, 4, prewarm=PREWARM_CFG4)
    sub = copy.copy(args)
    sub.no_cpu = True
    keep = ("value", "unit", "steps", "warmup", "ms_per_step", "config", "roofline", "roofline_hbm", "roofline_c54", "phase_ms_per_step")

    def nested(res):
        return {k: res[k] for k in keep if k in res}

    gc.collect(); torch.cuda.empty_cache()
    out["cold_start"] = nested(bench_net(sub, 4, cold=True))
    gc.collect(); torch.cuda.empty_cache()
    sub.steps, sub.warmup = 5, 2
    out["calc_only"] = nested(bench_calc(sub, 4))
    gc.collect(); torch.cuda.empty_cache()
    sub.steps, sub.warmup, sub.calibrate_copy = 10, 3, False
    out["server_config1"] = nested(bench_server(sub))
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="all")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg (profiling runs)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run plain 240 MB device copies (reference for rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (lambda learners are simulated on it); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    if args.workload == "all":
        out = bench_all(args)
    elif args.workload == "alex":
        out = bench_net(args, 4, prewarm=PREWARM_CFG4)
    elif args.workload == "alex-cold":
        out = bench_net(args, 4, cold=True)
    elif args.workload == "server":
        out = bench_server(args)
    elif args.workload in ("cifar", "cifar-fp32-c4", "cifar-fp32-c1"):
        out = bench_net(args, {"cifar": 3, "cifar-fp32-c4": 0, "cifar-fp32-c1": 2}[args.workload])
    elif args.workload in ("cifar-calc", "alex-calc"):
        out = bench_calc(args, {"cifar-calc": 3, "alex-calc": 4}[args.workload])
    elif args.workload == "alex-calc-shared":      # all learners on one weight version (what 1-softsync would give)
        out = bench_calc(args, 4, shared=True)
    else:
        raise SystemExit("unknown workload " + args.workload)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
