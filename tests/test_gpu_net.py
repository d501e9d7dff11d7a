"""GPU parity of calcGradient and of whole n-softsync runs against the CPU oracle, through the C ABI.

Error measures.  (1) ||a - b||_2 / ||b||_2 over the whole flat vector and over each layer's weight and bias
tensor (the largest is checked).  Bounds: per gradient 1e-4 (fp32 compute) and 2e-2 (bf16 compute);
weights after K updates 1e-3 (fp32); timestamps and staleness exact.  (2) Element by element, so that one
wrong element of a large tensor (a ragged tile edge, a last row) cannot hide in a norm:
|a - b| <= tol (|b| + rms(b's tensor)) for EVERY element; tol is 1e-3 in fp32 and, in bf16 compute, the value stated
at each test (a wholly wrong element -- zero, garbage, a neighbour's value -- sits at about 1).

bf16 compute: a ReLU sign or a max-pool winner decided on a bfloat16 value can differ from the decision on
the exact value, and one flipped decision moves a whole term of a weight-gradient sum.  Such decisions are
therefore compared in the kernel's precision: the reference for bf16 runs is the oracle's reduced-precision
mode (same rounding points, sums in fp64).  Against the exact oracle the 2e-2 bound is checked where the
sums are long enough for flips to average out (the mu = 128 configuration), and reported otherwise.
"""
import os

import numpy as np
import pytest

import workloads as wl
from oracle import cnn, protocol

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = {"fp32": 1e-4, "bf16": 2e-2}
ELEM_TOL = {"fp32": 1e-3, "bf16": 0.25}       # element-wise bound; bf16: single elements carry up to a few bf16 roundings


def rel(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    nb = np.linalg.norm(b)
    return np.linalg.norm(a - b) / nb if nb > 0 else np.linalg.norm(a)


def layer_errors(net, g, ref):
    """Largest relative error over the whole vector and each weight / bias tensor."""
    errs = [rel(g, ref)]
    pos = 0
    for ws, nb in wl.param_shapes(net):
        nw = int(np.prod(ws))
        errs.append(rel(g[pos:pos + nw], ref[pos:pos + nw]))
        pos += nw
        errs.append(rel(g[pos:pos + nb], ref[pos:pos + nb]))
        pos += nb
    assert pos == g.size
    return max(errs), errs


def elem_error(net, g, ref):
    """Largest |a - b| / (|b| + rms(b's tensor)) over all elements, and where it is."""
    g = np.asarray(g, np.float64)
    ref = np.asarray(ref, np.float64)
    worst, where = 0.0, None
    pos = 0
    for ws, nb in wl.param_shapes(net):
        for n in (int(np.prod(ws)), nb):
            b = ref[pos:pos + n]
            rms = np.sqrt(np.mean(b * b))
            if rms > 0:
                r = np.abs(g[pos:pos + n] - b) / (np.abs(b) + rms)
                k = int(np.argmax(r))
                if r[k] > worst:
                    worst, where = float(r[k]), pos + k
            pos += n
    return worst, where


def draw_case(net, lam, mu, seed, scale):
    rng = np.random.default_rng(seed)
    theta = (rng.standard_normal(wl.num_params(net)) * scale).astype(np.float32)
    return theta, wl.images(net, lam * mu, seed + 1), wl.labels(net, lam * mu, seed + 2)


MIN_MARGIN = 2e-7
SPREAD_FACTOR = 1.5     # a GPU tensor may lie this much further from the oracle than the oracle's own evaluations lie apart


def decided_seed(net, lam, mu, seed, scale, tries=16):
    """The first seed of seed, seed + 1, ... whose case has every ReLU input decided at fp32 precision: the oracle's
    smallest |ReLU input| / sum |its terms| is at least MIN_MARGIN.  Below that the sign of some ReLU input depends on
    the order of an fp32 sum, the 1e-4 bound has no meaning for the case (one flipped ReLU moves early-layer gradients
    by 1e-3), and the case is passed over -- by the oracle's number, never by a GPU result.
    MIN_MARGIN = 2e-7 is three float roundings (2^-24 each) of the whole term sum.  An fp32 accumulation of K terms is
    off by about sqrt(K) roundings of ONE term, i.e. 2^-24 / sqrt(K) of the term sum: below 1e-8 for the K <= 6 400 of
    these nets (the flips that were seen sat at 6e-9 and 2e-8), so the margin leaves a factor of ten.  The largest test
    net has 280 000 ReLU inputs per case, whose smallest margin is typically 1e-6: a larger threshold would pass over
    nearly every draw."""
    for s in range(seed, seed + tries):
        theta, X, _ = draw_case(net, lam, mu, s, scale)
        m = min(cnn.min_relu_margin(net, theta, X[L * mu:(L + 1) * mu]) for L in range(lam))
        if m >= MIN_MARGIN:
            if s != seed:
                print("seed %d -> %d: a ReLU input of the drawn case lies within %.1e of its terms' magnitude" % (seed, s, MIN_MARGIN))
            return s
    pytest.skip("no drawn case with every ReLU input decided at fp32 precision (margin %.1e)" % MIN_MARGIN)


def one_gradient(net, mu, compute, seed, scale=0.3, lam=2, exact=False, both=False):
    """calcGradient of `lam` learners with different batches on the same weights vs the oracle.
    both: also return the exact oracle's gradient (bf16 runs are judged against the reduced-precision mode and
    reported against the exact one)."""
    from paper_1511_05950_amd import binding
    P = wl.num_params(net)
    theta, X, Y = draw_case(net, lam, mu, seed, scale)
    Xd, Yd = torch.from_numpy(X).cuda(), torch.from_numpy(Y).cuda()
    ctx = binding.Sasgd(lam, mu, lam, 2, net=net, compute=compute, init_weights=theta)
    assert ctx.P == P
    loss = torch.zeros(lam, device="cuda")
    for L in range(lam):
        ctx.getMinibatch(L, Xd[L * mu:(L + 1) * mu], Yd[L * mu:(L + 1) * mu])
        assert ctx.pullWeights(L, 0) == 0
    ctx.calcGradient(list(range(lam)), loss)
    out = []
    for L in range(lam):
        g = ctx.copyGradient(L)
        rl, rg = cnn.loss_and_gradient(net, theta, X[L * mu:(L + 1) * mu], Y[L * mu:(L + 1) * mu],
                                       round_bf16=(compute == "bf16" and not exact))
        if both:
            _, eg = cnn.loss_and_gradient(net, theta, X[L * mu:(L + 1) * mu], Y[L * mu:(L + 1) * mu])
            out.append((g, rg, float(loss[L].item()), rl, eg))
        else:
            out.append((g, rg, float(loss[L].item()), rl))
    ctx.destroy()
    return out


def check_gradient(net, compute, g, rg, loss, rl, tag, elem_tol=None):
    worst, errs = layer_errors(net, g, rg)
    assert worst < TOL[compute], (tag, compute, errs)
    ew, at = elem_error(net, g, rg)
    assert ew < (ELEM_TOL[compute] if elem_tol is None else elem_tol), (tag, compute, "element", at, ew)
    assert abs(loss - rl) < (1e-5 if compute == "fp32" else 2e-2) * max(1.0, abs(rl))
    return worst, ew


TINY = {
    "max_clipped": wl.tiny_net(3, 9, 7, 5, conv=((4, 3, 1, 1),), pool="maxpool"),
    "avg_clipped": wl.tiny_net(2, 8, 8, 3, conv=((3, 3, 1, 0),), pool="avgpool"),
    "stride2_pad": wl.tiny_net(3, 11, 10, 4, conv=((4, 5, 2, 2), (5, 3, 1, 1)), pool="avgpool", fc_hidden=6),
    "two_conv_max": wl.tiny_net(2, 12, 12, 3, conv=((3, 3, 1, 1), (4, 3, 1, 0)), pool="maxpool", fc_hidden=7),
    "stride4_nopad": wl.tiny_net(3, 23, 23, 4, conv=((5, 11, 4, 0),), pool="maxpool"),
    "wide": wl.tiny_net(5, 17, 13, 11, conv=((37, 3, 1, 1), (70, 3, 1, 1)), pool="maxpool", fc_hidden=33),
    # shapes the bf16 MFMA kernels take (channel counts multiples of 8), with ragged tile edges
    "mfma_pad3": wl.tiny_net(3, 13, 11, 8, conv=((16, 3, 1, 1), (24, 5, 1, 2)), pool="maxpool", fc_hidden=40),
    "mfma_s2d": wl.tiny_net(3, 29, 27, 16, conv=((8, 7, 2, 0), (72, 3, 1, 0)), pool="avgpool", fc_hidden=136),
    # windows over multiples of 32 channels (input patch kept in LDS): tiles spanning several images, ragged last
    # tile, 1 / 3 / 5 / 8 channel chunks, odd and even tap counts, both tile widths, forward and input gradient
    "patch_3x3": wl.tiny_net(3, 9, 8, 8, conv=((32, 3, 1, 1), (96, 3, 1, 1), (128, 3, 1, 0), (96, 2, 1, 1)), pool="maxpool", fc_hidden=24),
    "patch_5x5": wl.tiny_net(3, 10, 9, 8, conv=((64, 3, 1, 1), (256, 5, 1, 2), (160, 3, 1, 1), (256, 4, 1, 1)), pool="avgpool", fc_hidden=24),
    # 16 and 48 input channels with 5 x 5 and 4 x 4 windows: the patch kernel that walks the filters' 16-k blocks
    "patch_c16": wl.tiny_net(3, 12, 11, 8, conv=((16, 3, 1, 1), (48, 5, 1, 2), (96, 4, 1, 1), (40, 5, 1, 2)), pool="maxpool", fc_hidden=24),
    "mfma_s4": wl.tiny_net(3, 39, 39, 8, conv=((24, 11, 4, 0), (40, 3, 1, 1), (136, 3, 1, 1)), pool="maxpool", fc_hidden=264),
}


@pytest.mark.parametrize("compute", ["fp32", "bf16"])
@pytest.mark.parametrize("name", sorted(TINY))
def test_tiny_net_gradient(name, compute):
    net = TINY[name]
    seed = sum(map(ord, name))
    if compute == "fp32":
        seed = decided_seed(net, 2, 3, seed, 0.3)
    for (g, rg, loss, rl, eg) in one_gradient(net, 3, compute, seed=seed, both=True):
        worst, ew = check_gradient(net, compute, g, rg, loss, rl, name)
        if compute == "bf16":           # reported, not asserted: the distance to the exact oracle (bf16 rounding of every tensor)
            print("%s bf16: vs reduced-precision oracle %.1e (element %.1e), vs exact oracle %.1e" % (name, worst, ew, layer_errors(net, g, eg)[0]))
        else:
            print("%s fp32: vs oracle %.1e (element %.1e)" % (name, worst, ew))


@pytest.mark.parametrize("compute,mu", [("fp32", 4), ("bf16", 4), ("bf16", 128)])
def test_cifar3_gradient(compute, mu):
    net = wl.CIFAR3
    for (g, rg, loss, rl) in one_gradient(net, mu, compute, seed=3, scale=0.05):
        worst, errs = layer_errors(net, g, rg)
        print(compute, mu, "per-layer relative errors:", ["%.2e" % e for e in errs])
        check_gradient(net, compute, g, rg, loss, rl, "cifar3 mu=%d" % mu)


def test_cifar3_bf16_against_exact_oracle():
    # config 3's shape (mu = 128): bf16 compute against the exact (unrounded) oracle
    net = wl.CIFAR3
    for (g, rg, loss, rl) in one_gradient(net, 128, "bf16", seed=3, scale=0.05, exact=True):
        worst, errs = layer_errors(net, g, rg)
        print("bf16 vs exact oracle, whole gradient then per-layer relative errors:", ["%.2e" % e for e in errs])
        assert errs[0] < 2e-2, errs          # the whole gradient, the quantity the bound is stated for
        assert worst < 5e-2, errs            # per tensor: conv1 (behind the max-pool) sits near 2e-2


def run_config(cfgd, compute=None, K=None):
    from paper_1511_05950_amd import binding, driver
    net, lam, mu, n = cfgd["net"], cfgd["lam"], cfgd["mu"], cfgd["n"]
    compute = compute or cfgd["compute"]
    sched = cfgd["schedule"]()
    if K is not None:
        sched = sched[:K]
    K = len(sched)
    R = int(sched.max()) + 1
    X, Y, w0 = cfgd["images"](), cfgd["labels"](), cfgd["weights"]()
    Xd, Yd = torch.from_numpy(X).cuda(), torch.from_numpy(Y).cuda()
    ctx = binding.Sasgd(lam, mu, n, R, net=net, compute=compute, lr_mode=cfgd["lr_mode"], alpha0=cfgd["alpha0"],
                        momentum=cfgd["momentum"], weight_decay=cfgd["weight_decay"], init_weights=w0)
    log = driver.run_softsync(ctx, sched, lambda i, l: (Xd[wl.batch_slice(cfgd, i, l)], Yd[wl.batch_slice(cfgd, i, l)]), lam)
    w = ctx.copyWeights()
    v = ctx.copyMomentum()
    assert ctx.timestamp() == K
    ctx.destroy()
    ref = protocol.run(cnn.make_callback(net), w0, lambda i, l: (X[wl.batch_slice(cfgd, i, l)], Y[wl.batch_slice(cfgd, i, l)]),
                       sched, lam, n, cfgd["alpha0"], cfgd["momentum"], cfgd["weight_decay"], cfgd["lr_mode"], keep=R)
    return w, v, log, ref


def test_config0_end_to_end():
    cfgd = wl.config(0)
    w, v, log, ref = run_config(cfgd)
    assert log == ref["log"]                                # timestamps and staleness bit-exact
    worst, errs = layer_errors(cfgd["net"], w, ref["theta"])
    assert worst < 1e-3, errs
    # the update itself (theta_K - theta_0) must match too, not only the weights it is added to
    w0 = cfgd["weights"]()
    assert rel(w - w0, ref["theta"] - w0) < 1e-3


def test_config2_200_updates():
    cfgd = wl.config(2)
    w, v, log, ref = run_config(cfgd)
    assert log == ref["log"]
    worst, errs = layer_errors(cfgd["net"], w, ref["theta"])
    assert worst < 1e-3, errs
    w0 = cfgd["weights"]()
    assert rel(w - w0, ref["theta"] - w0) < 1e-3
    assert rel(v, ref["v"]) < 1e-3


@pytest.mark.parametrize("mode", ["per_gradient", "mean_staleness"])
def test_config3_first_updates(mode):
    """BASELINE config 3 as bench.py runs it (CIFAR-shaped, bf16 compute, lambda = 18 learners of mu = 128 in one batched
    call, 1-softsync: c = 18 gradients averaged per update, staleness in {0, 1, 2}), its first two updates, in both
    readings of its learning rate (per gradient, and one rate per update from the mean staleness), against the
    oracle's reduced-precision mode and its exact mode."""
    from paper_1511_05950_amd import binding, driver
    cfgd = wl.config(3)
    net, lam, mu, n, c = cfgd["net"], cfgd["lam"], cfgd["mu"], cfgd["n"], cfgd["c"]
    K = 2
    sched = cfgd["schedule"]()[:K]
    X, Y, w0 = wl.images(net, K * c * mu, 7), wl.labels(net, K * c * mu, 8), cfgd["weights"]()
    Xd, Yd = torch.from_numpy(X).cuda(), torch.from_numpy(Y).cuda()
    sl = lambda i, l: slice((i * c + l) * mu, (i * c + l + 1) * mu)
    ctx = binding.Sasgd(lam, mu, n, 3, net="cifar3", compute="bf16", lr_mode=mode, alpha0=cfgd["alpha0"], momentum=cfgd["momentum"],
                        weight_decay=cfgd["weight_decay"], init_weights=w0)
    log = driver.run_softsync(ctx, sched, lambda i, l: (Xd[sl(i, l)], Yd[sl(i, l)]), lam)
    w, v = ctx.copyWeights(), ctx.copyMomentum()
    ctx.destroy()
    refs = {}
    for reduced in (True, False):
        refs[reduced] = protocol.run(cnn.make_callback(net, round_bf16=reduced), w0, lambda i, l: (X[sl(i, l)], Y[sl(i, l)]), sched, lam, n,
                                     cfgd["alpha0"], cfgd["momentum"], cfgd["weight_decay"], mode)
    # The update is the average of 18 (then 36) gradients of random-label mini-batches: what is particular to a mini-batch
    # averages out, the error of rounding the SHARED weights and activations to bf16 does not, so the update's distance to
    # the exact oracle is several times a single gradient's.  The bound is the stated 2e-2 against the reduced-precision
    # oracle, and against the exact one SPREAD_FACTOR times the distance between the oracle's own two modes where
    # that exceeds 2e-2.
    _, own = layer_errors(net, refs[True]["theta"] - w0, refs[False]["theta"] - w0)
    for reduced in (True, False):
        ref = refs[reduced]
        assert log == ref["log"]
        assert [t for (_, _, _, _, t) in log[:c]] == [0] * c      # every first-update gradient reads theta_0
        worst, errs = layer_errors(net, w - w0, ref["theta"] - w0)
        tol = [2e-2] * len(errs) if reduced else [max(2e-2, SPREAD_FACTOR * e) for e in own]
        print("config 3 (%s), 2 updates, update vs %s oracle:" % (mode, "reduced-precision" if reduced else "exact"), ["%.1e" % e for e in errs])
        if not reduced:
            print("   oracle's reduced-precision mode vs its exact mode:", ["%.1e" % e for e in own])
        assert all(e < t for e, t in zip(errs, tol)), (errs, tol)
        assert rel(v, ref["v"]) < tol[0]


def test_config3_all_100_updates():
    """BASELINE config 3 in full: 100 updates of c = 18 gradients (1 800 mini-batches of 128 images) through the
    batched driver.  The bookkeeping log must equal the oracle's exactly; the update theta_100 - theta_0 and the momentum
    are compared, whole and per tensor, with the oracle's two runs stored in tests/golden/config3_run.npz (written by
    tests/golden/make_config_runs.py from the oracle alone): 2e-2 against the reduced-precision mode; against the exact
    mode 2e-2 where the distance between the oracle's own two runs allows it, SPREAD_FACTOR times that distance elsewhere
    (see test_config3_first_updates)."""
    from paper_1511_05950_amd import binding, driver
    gold = np.load(os.path.join(GOLDEN, "config3_run.npz"))
    cfgd = wl.config(3)
    net, lam, mu, n = cfgd["net"], cfgd["lam"], cfgd["mu"], cfgd["n"]
    sched = cfgd["schedule"]()
    X, Y, w0 = cfgd["images"](), cfgd["labels"](), cfgd["weights"]()
    Xd, Yd = torch.from_numpy(X).cuda(), torch.from_numpy(Y).cuda()
    ctx = binding.Sasgd(lam, mu, n, int(sched.max()) + 1, net="cifar3", compute="bf16", lr_mode=cfgd["lr_mode"], alpha0=cfgd["alpha0"],
                        momentum=cfgd["momentum"], weight_decay=cfgd["weight_decay"], init_weights=w0)
    log, calls = driver.run_softsync_batched(ctx, sched, lambda i, l: (Xd[wl.batch_slice(cfgd, i, l)], Yd[wl.batch_slice(cfgd, i, l)]), lam)
    w, v = ctx.copyWeights(), ctx.copyMomentum()
    assert ctx.timestamp() == 100
    ctx.destroy()
    assert np.array_equal(np.asarray(log, dtype=np.int64), gold["log"])
    upd = w.astype(np.float64) - w0.astype(np.float64)
    _, own = layer_errors(net, gold["update_reduced"], gold["update_exact"])       # the oracle's two modes against each other
    print("config 3, 100 updates, oracle's reduced-precision run vs its exact run:", ["%.1e" % e for e in own])
    for tag in ("reduced", "exact"):
        worst, errs = layer_errors(net, upd, gold["update_" + tag])
        ev = rel(v, gold["v_" + tag])
        tol = [2e-2] * len(errs) if tag == "reduced" else [max(2e-2, SPREAD_FACTOR * e) for e in own]
        print("config 3, 100 updates vs %s oracle run: update" % tag, ["%.1e" % e for e in errs], "momentum %.1e" % ev)
        assert all(e < t for e, t in zip(errs, tol)), (tag, errs, tol)
        assert ev < tol[0], (tag, ev)


def test_batched_driver_matches_plain_driver():
    # merging calcGradient calls across updates must not change versions, staleness or (up to summation order) weights
    from paper_1511_05950_amd import binding, driver
    cfgd = wl.config(2)
    net, lam, mu, n = cfgd["net"], cfgd["lam"], cfgd["mu"], cfgd["n"]
    sched = cfgd["schedule"]()[:60]
    X, Y, w0 = cfgd["images"](), cfgd["labels"](), cfgd["weights"]()
    Xd, Yd = torch.from_numpy(X).cuda(), torch.from_numpy(Y).cuda()
    bo = lambda i, l: (Xd[wl.batch_slice(cfgd, i, l)], Yd[wl.batch_slice(cfgd, i, l)])
    out = []
    for batched in (False, True):
        ctx = binding.Sasgd(lam, mu, n, int(sched.max()) + 1, net=net, alpha0=cfgd["alpha0"], momentum=cfgd["momentum"], init_weights=w0)
        if batched:
            log, calls = driver.run_softsync_batched(ctx, sched, bo, lam)
            assert calls < len(sched)
        else:
            log = driver.run_softsync(ctx, sched, bo, lam)
        out.append((log, ctx.copyWeights()))
        ctx.destroy()
    assert out[0][0] == out[1][0]
    assert rel(out[1][1] - w0, out[0][1] - w0) < 1e-5


def cosine(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    return float(a @ b / (np.linalg.norm(a) * np.linalg.norm(b)))


GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def alex8_spread():
    """Per-tensor spread between CPU evaluations of the AlexNet-shaped bf16 gradient, measured with the oracle alone
    (tests/golden/make_alex8_bf16_spread.py): name -> (|R-E|/|E|, |R32-R|/|R|, |R32-E|/|E|), E the exact oracle, R its
    reduced-precision mode, R32 the reduced-precision mode with float running sums."""
    rows = {}
    for line in open(os.path.join(GOLDEN, "alex8_bf16_spread.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, a, b, c = line.split()
        rows[name] = (float(a), float(b), float(c))
    return rows


def alex8_tensor_names():
    return ["whole"] + [n + s for n in ("conv1", "conv2", "conv3", "conv4", "conv5", "fc6", "fc7", "fc8") for s in (".w", ".b")]



def alex8_tolerances():
    """Bound per tensor (order of layer_errors) against the reduced-precision oracle and against the exact one: the
    stated 2e-2 wherever the CPU-measured spread allows it, SPREAD_FACTOR times that spread elsewhere."""
    sp = alex8_spread()
    vs_reduced = [max(2e-2, SPREAD_FACTOR * sp[n][1]) for n in alex8_tensor_names()]
    vs_exact = [max(2e-2, SPREAD_FACTOR * sp[n][0]) for n in alex8_tensor_names()]
    return vs_reduced, vs_exact


def learners_on_versions(net, netarg, w0, X, Y, ver_of, push_seed=0, mu=None):
    """calcGradient of len(ver_of) learners in ONE call, learner k on weight version ver_of[k].  Versions 1, 2, ... are
    made from w0 by server updates with seeded random gradients.  Returns the gradients, the losses and, per learner,
    the weights it read (as the library holds them)."""
    from paper_1511_05950_amd import binding
    lam = len(ver_of)
    mu = X.shape[0] // lam if mu is None else mu
    versions = max(ver_of) + 1
    ctx = binding.Sasgd(max(lam, 2), mu, max(lam, 2), versions, net=netarg, compute="bf16", alpha0=0.5, init_weights=w0)
    rng = np.random.default_rng(push_seed)
    scale = 0.2 * float(np.sqrt(np.mean(np.asarray(w0, dtype=np.float64) ** 2)))
    for _ in range(versions - 1):
        push = torch.from_numpy((rng.standard_normal(ctx.P) * scale).astype(np.float32)).cuda()
        ctx.pushGradientExternal(push, ctx.timestamp())
        ctx.sumGradients()
        ctx.applyUpdate()
        torch.cuda.synchronize()
        del push
    Xd, Yd = torch.from_numpy(X).cuda(), torch.from_numpy(Y).cuda()
    loss = torch.zeros(lam, device="cuda")
    ids = list(range(lam)) if lam > 1 else [1]
    for k, L in enumerate(ids):
        ctx.getMinibatch(L, Xd[k * mu:(k + 1) * mu], Yd[k * mu:(k + 1) * mu])
        assert ctx.pullWeights(L, ctx.timestamp() - ver_of[k]) == ver_of[k]
    ctx.calcGradient(ids, loss)
    grads = [ctx.copyGradient(L) for L in ids]
    weights = {j: ctx.copyWeights(j) for j in sorted(set(ver_of))}
    ctx.destroy()
    return grads, [float(v) for v in loss.cpu()], [weights[j] for j in ver_of]


def alex_learners(net, netarg, w0, X, Y, versions=1, lam=1, push_seed=0):
    """`lam` learners in one call at mu = len(X) / lam, learner L on weight version L * versions // lam."""
    return learners_on_versions(net, netarg, w0, X, Y, [k * versions // lam for k in range(lam)], push_seed)


def test_alex8_shapes_smooth_variant_full_size():
    """Every kernel of config 4 at its real shape (mu = 16, 3x224x224, 62.4 M parameters) on the decision-free
    variant of the network (no ReLU, average pooling): bf16 compute must match the oracle to 2e-2 per tensor, and
    element by element."""
    net = wl.ALEX8_SMOOTH
    w0 = wl.init_weights(net, wl.SEED0 + 4002, std=0.02)
    X, Y = wl.images(net, 16, 77), wl.labels(net, 16, 78)
    (g,), (loss,), _ = alex_learners(net, net, w0, X, Y)
    rl, rg = cnn.loss_and_gradient(net, w0, X, Y, round_bf16=True)
    worst, errs = layer_errors(net, g, rg)
    ew, at = elem_error(net, g, rg)
    print("alex8_smooth bf16 vs reduced-precision oracle:", ["%.1e" % e for e in errs], "element-wise %.2e" % ew)
    assert worst < 2e-2, errs
    assert ew < ELEM_TOL["bf16"], (at, ew)
    el, eg = cnn.loss_and_gradient(net, w0, X, Y)
    worst, errs = layer_errors(net, g, eg)
    ew, at = elem_error(net, g, eg)
    print("alex8_smooth bf16 vs exact oracle:", ["%.1e" % e for e in errs], "element-wise %.2e" % ew)
    assert worst < 2e-2, errs
    assert ew < ELEM_TOL["bf16"], (at, ew)
    assert abs(loss - el) < 1e-3 * abs(el)


def test_alex8_gradient_full_size():
    """One learner step of BASELINE config 4 at full size.  With ReLU and max pooling in an eight-layer net whose
    initial weights leave every pre-activation near zero, a bf16 gradient is reproducible only to a few per cent by ANY
    two evaluations: storing a tensor in bf16 moves values by 2^-9, the differences spread to every later activation
    within two layers, and a share of the ReLU signs and pooling winners comes out differently; each flip moves a
    whole term of a weight-gradient sum.  tests/golden/alex8_bf16_spread.txt has the CPU evidence (oracle only): its
    exact mode, its reduced-precision mode and that mode with float running sums lie 3 - 24 % apart per tensor on this
    very case.  The bound per tensor is the stated 2e-2 where that spread allows it (the last layer, with no decision
    between it and the loss) and SPREAD_FACTOR times the spread elsewhere; the loss must match to 1e-5."""
    net = wl.ALEX8
    cfgd = wl.config(4)
    w0 = cfgd["weights"]()
    X, Y = wl.images(net, cfgd["mu"], 77), wl.labels(net, cfgd["mu"], 78)
    (g,), (loss,), _ = alex_learners(net, "alex8", w0, X, Y)
    tol_r, tol_e = alex8_tolerances()
    rl, rg = cnn.loss_and_gradient(net, w0, X, Y, round_bf16=True)
    worst, errs = layer_errors(net, g, rg)
    print("alex8 bf16 vs reduced-precision oracle:", ["%.1e" % e for e in errs])
    print("                          bounds      :", ["%.1e" % e for e in tol_r])
    assert abs(loss - rl) < 1e-5 * abs(rl)
    assert all(e < t for e, t in zip(errs, tol_r)), (errs, tol_r)
    assert tol_r[-2] == 2e-2 and tol_r[-1] == 2e-2            # fc8 weights and bias stay at the stated bound
    assert cosine(g, rg) > 0.995
    el, eg = cnn.loss_and_gradient(net, w0, X, Y)
    worst, errs = layer_errors(net, g, eg)
    print("alex8 bf16 vs exact oracle            :", ["%.1e" % e for e in errs], "cosine %.5f" % cosine(g, eg))
    print("                          bounds      :", ["%.1e" % e for e in tol_e])
    assert all(e < t for e, t in zip(errs, tol_e)), (errs, tol_e)
    assert cosine(g, eg) > 0.995


def test_alex8_six_learners_on_three_versions_full_size():
    """The situation bench.py times at full size: several learners of ONE batched call, each pair on a weight version
    of its own (lambda-softsync), which switches the convolution kernels to their XCD-contiguous tile order and 256-row
    tiles.  Every learner's gradient against the oracle on the weights that learner read: element by element on the
    decision-free variant, at the spread-derived per-tensor bounds on the network itself (one learner per version)."""
    mu, lam, versions = 16, 6, 3
    net = wl.ALEX8_SMOOTH
    w0 = wl.init_weights(net, wl.SEED0 + 4002, std=0.02)
    X, Y = wl.images(net, lam * mu, 81), wl.labels(net, lam * mu, 82)
    grads, losses, weights = alex_learners(net, net, w0, X, Y, versions=versions, lam=lam, push_seed=83)
    assert rel(weights[2], weights[0]) > 1e-2 and rel(weights[4], weights[2]) > 1e-2     # the versions do differ
    for L in range(lam):
        print("smooth variant, learner %d" % L, flush=True)
        rl, rg = cnn.loss_and_gradient(net, weights[L], X[L * mu:(L + 1) * mu], Y[L * mu:(L + 1) * mu], round_bf16=True)
        worst, errs = layer_errors(net, grads[L], rg)
        ew, at = elem_error(net, grads[L], rg)
        assert worst < 2e-2, (L, errs)
        assert ew < ELEM_TOL["bf16"], (L, at, ew)
        assert abs(losses[L] - rl) < 1e-3 * abs(rl)
    net = wl.ALEX8
    w0 = wl.config(4)["weights"]()
    grads, losses, weights = alex_learners(net, "alex8", w0, X, Y, versions=versions, lam=lam, push_seed=84)
    tol_r, _ = alex8_tolerances()
    for L in (1, 2, 5):                                       # one learner of every version
        print("alex8, learner %d" % L, flush=True)
        rl, rg = cnn.loss_and_gradient(net, weights[L], X[L * mu:(L + 1) * mu], Y[L * mu:(L + 1) * mu], round_bf16=True)
        worst, errs = layer_errors(net, grads[L], rg)
        print("   ", ["%.1e" % e for e in errs])
        assert abs(losses[L] - rl) < 1e-5 * abs(rl)
        assert all(e < t for e, t in zip(errs, tol_r)), (L, errs, tol_r)


def sample_rel(a, b):
    nb = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / nb) if nb > 0 else float(np.linalg.norm(a))


def test_config4_all_20_updates():
    """BASELINE config 4 in full, as bench.py runs it (AlexNet-shaped, bf16, 18-softsync, ring of 37 versions, batched
    driver): all 20 updates.  Bookkeeping must equal the oracle's log exactly.  The update theta_20 - theta_0 is compared
    with the oracle's runs (tests/golden/config4_run.npz, written by tests/golden/make_config_runs.py from the oracle
    alone) on the stored sample of every tensor -- its edges and 16 384 seeded draws.  Over 20 updates two bf16
    evaluations drift further apart than on one gradient (the second evaluates its later gradients on slightly different
    weights), so the bounds come from the oracle's own runs of the same 20 updates: against the reduced-precision run
    SPREAD_FACTOR times the distance between that run and the run with float running sums, against the exact run
    SPREAD_FACTOR times the distance between the reduced-precision and the exact run, never below the stated 2e-2."""
    from paper_1511_05950_amd import binding, driver
    gold = np.load(os.path.join(GOLDEN, "config4_run.npz"))
    cfgd = wl.config(4)
    net, lam, mu, n = cfgd["net"], cfgd["lam"], cfgd["mu"], cfgd["n"]
    sched = cfgd["schedule"]()
    X, Y, w0 = cfgd["images"](), cfgd["labels"](), cfgd["weights"]()
    Xd, Yd = torch.from_numpy(X).cuda(), torch.from_numpy(Y).cuda()
    ctx = binding.Sasgd(lam, mu, n, 37, net="alex8", compute="bf16", alpha0=cfgd["alpha0"], momentum=cfgd["momentum"],
                        weight_decay=cfgd["weight_decay"], init_weights=w0)
    log, calls = driver.run_softsync_batched(ctx, sched, lambda i, l: (Xd[wl.batch_slice(cfgd, i, l)], Yd[wl.batch_slice(cfgd, i, l)]), lam)
    w = ctx.copyWeights()
    old = ctx.copyWeights(len(sched) - 1)             # bf16 copy of the previous version, from the ring
    assert ctx.timestamp() == len(sched)
    ctx.destroy()
    assert np.array_equal(np.asarray(log, dtype=np.int64), gold["log"])          # timestamps, staleness, learners: exact
    versions = sorted({int(j) for (_, _, _, j, _) in log})
    print("batched calls %d, weight versions read: %s" % (calls, versions))
    assert len(versions) > 1                          # stale ring slots other than theta_0 are read at full size
    assert np.all((old.view(np.uint32) & 0xFFFF) == 0)
    idx = gold["idx"].astype(np.int64)
    upd = (w.astype(np.float64) - w0.astype(np.float64))[idx]
    # sample positions per tensor, in the order of the stored sample
    bounds, pos = [], 0
    for ws, nb in wl.param_shapes(net):
        for cnt in (int(np.prod(ws)), nb):
            bounds.append((pos, pos + cnt))
            pos += cnt

    def per_tensor(a, b):
        out = [sample_rel(a, b)]
        for (lo, hi) in bounds:
            sel = (idx >= lo) & (idx < hi)
            out.append(sample_rel(a[sel], b[sel]))
        return out

    run_e, run_r, run_r32 = (gold[k].astype(np.float64) for k in ("update_exact", "update_reduced", "update_r32"))
    own = {"reduced": per_tensor(run_r32, run_r), "exact": per_tensor(run_r, run_e)}
    for tag, ref in (("reduced", run_r), ("exact", run_e)):
        errs = per_tensor(upd, ref)
        tol = [max(2e-2, SPREAD_FACTOR * e) for e in own[tag]]
        print("config 4, update after 20 steps vs %s oracle run:" % tag, ["%.1e" % e for e in errs], "cosine %.5f" % cosine(upd, ref))
        print("   the oracle's own runs apart (%s):" % ("float sums vs reduced" if tag == "reduced" else "reduced vs exact"), ["%.1e" % e for e in own[tag]])
        assert all(e < t for e, t in zip(errs, tol)), (tag, errs, tol)
        assert cosine(upd, ref) > 0.995


def test_learner_protocol_errors():
    from paper_1511_05950_amd import binding
    net = TINY["avg_clipped"]
    P = wl.num_params(net)
    ctx = binding.Sasgd(3, 2, 3, 2, net=net, init_weights=np.zeros(P, np.float32))
    X = torch.zeros(2, *net["input"], device="cuda")
    Y = torch.zeros(2, dtype=torch.int32, device="cuda")
    with pytest.raises(binding.SasgdError) as e:
        ctx.calcGradient([0])                              # nothing bound
    assert e.value.code == binding.ESTATE
    ctx.getMinibatch(0, X, Y)
    with pytest.raises(binding.SasgdError) as e:
        ctx.calcGradient([0])                              # no weights pulled
    assert e.value.code == binding.ESTATE
    with pytest.raises(binding.SasgdError) as e:
        ctx.pushGradient(0)                                # nothing computed
    assert e.value.code == binding.ESTATE
    ctx.pullWeights(0, 5)                                  # clamped to version 0
    with pytest.raises(binding.SasgdError) as e:
        ctx.calcGradient([0, 0])
    assert e.value.code == binding.EINVAL
    ctx.calcGradient([0])
    assert ctx.gradientTimestamp(0) == 0
    assert ctx.pushGradient(0) == 0
    with pytest.raises(binding.SasgdError) as e:
        ctx.pushGradient(0)                                # already pushed
    assert e.value.code == binding.ESTATE
    ctx.getMinibatch(0, X, Y)
    ctx.pullWeights(0, 0)
    with pytest.raises(binding.SasgdError) as e:
        ctx.calcGradient([0])                              # previous gradient still pending
    assert e.value.code == binding.ESTATE
    ctx.sumGradients()
    assert ctx.applyUpdate() == 1
    # learner 1 pulls version 0 (staleness 1), then two more updates would evict it from a ring of depth 2
    ctx.getMinibatch(1, X, Y)
    assert ctx.pullWeights(1, 1) == 0
    ctx.calcGradient([0])
    assert ctx.pushGradient(0) == 1                        # computed on version 0, pushed at timestamp 1
    ctx.sumGradients()
    with pytest.raises(binding.SasgdError) as e:
        ctx.applyUpdate()                                  # would overwrite version 0, still held by learner 1
    assert e.value.code == binding.ERANGE
    ctx.calcGradient([1])
    assert ctx.applyUpdate() == 2
    with pytest.raises(binding.SasgdError) as e:
        ctx.pullWeights(2, 0) and ctx.copyWeights(0)       # version 0 has left the ring
    assert e.value.code == binding.ERANGE
    ctx.destroy()


def test_bad_labels_poison_the_loss_not_memory():
    from paper_1511_05950_amd import binding
    net = TINY["avg_clipped"]
    P = wl.num_params(net)
    ctx = binding.Sasgd(1, 2, 1, 1, net=net, init_weights=np.zeros(P, np.float32))
    X = torch.zeros(2, *net["input"], device="cuda")
    Y = torch.tensor([0, 99], dtype=torch.int32, device="cuda")
    loss = torch.zeros(1, device="cuda")
    ctx.getMinibatch(0, X, Y)
    ctx.pullWeights(0, 0)
    ctx.calcGradient([0], loss)
    assert torch.isnan(loss).all()
    ctx.destroy()


# ---------------------------------------------------------------------------------------------------------------
# Fully connected weight gradients kept as rank-mu factors (bf16 compute): the product is formed inside applyUpdate.
FC_NET = {"name": "fcnet", "input": (3, 10, 10), "classes": 8,
          "layers": [("conv", 8, 3, 1, 1), ("relu",), ("maxpool", 3, 2), ("fc", 72), ("relu",), ("fc", 24), ("relu",), ("fc", 8)]}


def _fc_run(flags, K=5):
    from paper_1511_05950_amd import binding, driver
    net, lam, n, mu = FC_NET, 6, 2, 5                      # c = 3 gradients per update, mu not a multiple of 8
    c = lam // n
    X = wl.images(net, K * c * mu, 70)
    Y = wl.labels(net, K * c * mu, 71)
    w0 = wl.init_weights(net, 72, std=0.1)
    Xd, Yd = torch.from_numpy(X).cuda(), torch.from_numpy(Y).cuda()
    sl = lambda i, l: slice((i * c + l) * mu, (i * c + l + 1) * mu)
    sched = wl.uniform_schedule(K, c, 0, 2, 73)
    ctx = binding.Sasgd(lam, mu, n, 3, net=net, compute="bf16", alpha0=0.05, momentum=0.9, weight_decay=1e-3, init_weights=w0, flags=flags)
    grads = []
    hook = lambda i, l, learner: grads.append(ctx.copyGradient(learner)) if i == 0 else None
    log = driver.run_softsync(ctx, sched, lambda i, l: (Xd[sl(i, l)], Yd[sl(i, l)]), lam, on_gradient=hook)
    out = dict(w=ctx.copyWeights(), v=ctx.copyMomentum(), grads=grads, log=log, factored=ctx.factoredParams(), w0=w0,
               X=X, Y=Y, sched=sched, sl=sl, net=net, lam=lam, n=n)
    ctx.destroy()
    return out


def test_factored_fc_gradient_matches_written_out_gradient_and_oracle():
    from paper_1511_05950_amd import binding
    fa = _fc_run(0)
    fl = _fc_run(binding.FLAG_FLAT_FC_GRADIENT)
    assert fa["factored"] == 72 * 200 + 24 * 72 + 8 * 24 and fl["factored"] == 0
    assert fa["log"] == fl["log"]
    # the first update's gradients are computed on identical weights: the expanded product equals the MFMA result
    for ga, gb in zip(fa["grads"], fl["grads"]):
        assert rel(ga, gb) < 1e-5
    # after K updates with momentum and decay the two runs differ by rounding only
    assert rel(fa["w"] - fa["w0"], fl["w"] - fl["w0"]) < 2e-3
    assert rel(fa["v"], fl["v"]) < 5e-3
    # and both follow the oracle (reduced-precision mode) within the bf16 bound
    net = fa["net"]
    ref = protocol.run(cnn.make_callback(net, round_bf16=True), fa["w0"], lambda i, l: (fa["X"][fa["sl"](i, l)], fa["Y"][fa["sl"](i, l)]),
                       fa["sched"], fa["lam"], fa["n"], 0.05, 0.9, 1e-3)
    assert fa["log"] == ref["log"]
    assert rel(fa["w"] - fa["w0"], ref["theta"] - fa["w0"]) < 2e-2


def test_factored_and_external_gradients_share_one_update():
    # one window of c = 2: a learner's gradient (factors) and a gradient pushed from outside (written out)
    from paper_1511_05950_amd import binding
    net, mu = FC_NET, 4
    X = wl.images(net, mu, 74)
    Y = wl.labels(net, mu, 75)
    w0 = wl.init_weights(net, 76, std=0.1)
    P = wl.num_params(net)
    gext = (np.random.default_rng(77).standard_normal(P) * 1e-2).astype(np.float32)
    Xd, Yd, Gd = torch.from_numpy(X).cuda(), torch.from_numpy(Y).cuda(), torch.from_numpy(gext).cuda()
    ctx = binding.Sasgd(2, mu, 1, 2, net=net, compute="bf16", alpha0=0.1, momentum=0.5, weight_decay=1e-2, init_weights=w0)
    assert ctx.factoredParams() > 0
    ctx.getMinibatch(0, Xd, Yd)
    ctx.pullWeights(0, 0)
    ctx.calcGradient([0])
    g0 = ctx.copyGradient(0)
    # an evaluation pass of the same learner on other images before the push must not disturb the saved factors
    X2 = torch.from_numpy(wl.images(net, mu, 78)).cuda()
    ctx.getMinibatch(0, X2, Yd)
    ctx.pullWeights(0, 0)
    ctx.evaluate([0], None, torch.zeros(mu, device="cuda", dtype=torch.int32))
    assert ctx.pushGradient(0) == 0
    assert ctx.pushGradientExternal(Gd, 0) == 0
    ctx.sumGradients()
    ctx.applyUpdate()
    w1, v1 = ctx.copyWeights(), ctx.copyMomentum()
    ctx.destroy()
    coef = 0.1 / 2
    v_ref = coef * g0.astype(np.float64) + coef * gext.astype(np.float64) + 2 * coef * 1e-2 * w0.astype(np.float64)
    assert rel(v1, v_ref) < 1e-5
    assert rel(w1 - w0, -v_ref) < 1e-5


def test_more_fully_connected_layers_than_the_factor_table_holds():
    # the layers past the table's size write their gradient out; the update must treat both kinds alike
    from paper_1511_05950_amd import binding
    layers = []
    for _ in range(18):
        layers += [("fc", 16), ("relu",)]
    net = {"name": "deepfc", "input": (8, 1, 1), "classes": 8, "layers": layers + [("fc", 8)]}
    mu = 4
    X = wl.images(net, mu, 80)
    Y = wl.labels(net, mu, 81)
    w0 = wl.init_weights(net, 82, std=0.35)
    Xd, Yd = torch.from_numpy(X).cuda(), torch.from_numpy(Y).cuda()
    res = []
    for flags in (0, binding.FLAG_FLAT_FC_GRADIENT):
        ctx = binding.Sasgd(1, mu, 1, 2, net=net, compute="bf16", alpha0=0.1, momentum=0.5, weight_decay=1e-2, init_weights=w0, flags=flags)
        fp = ctx.factoredParams()
        ctx.getMinibatch(0, Xd, Yd)
        ctx.pullWeights(0, 0)
        ctx.calcGradient([0])
        assert ctx.pushGradient(0) == 0
        ctx.sumGradients()
        ctx.applyUpdate()
        res.append((fp, ctx.copyWeights(), ctx.copyGradient(0)))
        ctx.destroy()
    # the layer on the raw input is not a candidate; the next 16 fill the table, the last two are written out
    assert res[0][0] == 16 * 16 * 16 and res[1][0] == 0
    assert np.abs(res[1][2]).max() > 0
    assert rel(res[0][2], res[1][2]) < 1e-5
    assert rel(res[0][1] - w0, res[1][1] - w0) < 1e-5


def test_learners_on_different_weight_versions_in_one_call():
    # two learners of one batched call hold different versions: every kernel must read each learner's own filters
    # (the convolution kernels also choose other tile shapes and another tile order in this case)
    from paper_1511_05950_amd import binding
    net, mu = TINY["patch_5x5"], 3
    rng = np.random.default_rng(90)
    P = wl.num_params(net)
    theta0 = (rng.standard_normal(P) * 0.3).astype(np.float32)
    X = wl.images(net, 2 * mu, 91)
    Y = wl.labels(net, 2 * mu, 92)
    Xd, Yd = torch.from_numpy(X).cuda(), torch.from_numpy(Y).cuda()
    push = torch.from_numpy((rng.standard_normal(P) * 0.5).astype(np.float32)).cuda()
    ctx = binding.Sasgd(2, mu, 2, 3, net=net, compute="bf16", alpha0=0.1, init_weights=theta0)
    ctx.getMinibatch(0, Xd[:mu], Yd[:mu])
    ctx.pullWeights(0, 0)
    ctx.pushGradientExternal(push, 0)
    ctx.sumGradients()
    ctx.applyUpdate()
    theta1 = ctx.copyWeights()
    assert rel(theta1, theta0) > 1e-2
    ctx.getMinibatch(1, Xd[mu:], Yd[mu:])
    ctx.pullWeights(1, 0)
    ctx.calcGradient([0, 1])
    for L, th in ((0, theta0), (1, theta1)):
        g = ctx.copyGradient(L)
        _, rg = cnn.loss_and_gradient(net, th, X[L * mu:(L + 1) * mu], Y[L * mu:(L + 1) * mu], round_bf16=True)
        worst, errs = layer_errors(net, g, rg)
        assert worst < TOL["bf16"], (L, errs)
    ctx.destroy()


GROUP_NETS = {
    # fully connected layers the grouped kernels take (inputs a multiple of 256): 1 024 -> 256 -> 24 (a ragged block of
    # units, a contraction of three chunks in the input gradient) behind a ReLU and a max pool
    "fc_256_24": wl.tiny_net(3, 9, 9, 24, conv=((64, 3, 1, 1),), pool="maxpool", fc_hidden=256),
    # the same shape family without a ReLU or a max pool (decision-free): checked element by element as well
    "fc_512_8_smooth": {"name": "tiny", "input": (3, 9, 9), "classes": 8,
                        "layers": [("conv", 64, 3, 1, 1), ("avgpool", 3, 2), ("fc", 512), ("fc", 8)]},
}


@pytest.mark.parametrize("mu,ver_of", [
    (16, [0, 1, 2, 2]),                          # a pair shares 32 rows: one row block
    (16, [1, 0, 1, 2, 1]),                       # three learners of one version, not next to each other: two row blocks
    (16, [0] * 8 + [1] * 3 + [2]),               # eight on one version: 128 rows, four row blocks per wavefront
    (16, [0] * 9 + [1] * 3 + [2]),               # nine on one version: groups of five and four
    (16, [0] * 18),                              # hardsync-like: three groups of six
    (16, [0] * 20 + [1, 1, 2]),                  # groups of seven, seven and six beside small ones
    (16, [1] * 32 + [0] * 2),                    # four full groups of eight
    (8, [0] * 64),                               # 64 learners on one version: four groups of sixteen 8-image members
    (4, [0] * 11 + [1, 1]),                      # mu = 4: eleven members make 44 rows
    (32, [0, 0, 0, 0, 0, 1]),                    # mu = 32: five members as groups of three and two
    (5, [0, 1, 0, 0]),                           # rows per member not a multiple of four
    (1, [0, 1, 0]),                              # single-image mini-batches: a group of two rows
])
@pytest.mark.parametrize("name", sorted(GROUP_NETS))
def test_fully_connected_layers_grouped_by_weight_version(name, mu, ver_of):
    """Learners of one batched call that read the same weight version share the reads of the fully connected weights
    (one launch per layer and direction, rows addressed through each member's workspace).  Every learner's gradient
    and loss against the oracle on the weights that learner read."""
    net = GROUP_NETS[name]
    smooth = not any(L[0] in ("relu", "maxpool") for L in net["layers"])
    lam = len(ver_of)
    rng = np.random.default_rng(770 + lam)
    w0 = (rng.standard_normal(wl.num_params(net)) * 0.05).astype(np.float32)
    X, Y = wl.images(net, lam * mu, 771), wl.labels(net, lam * mu, 772)
    grads, losses, weights = learners_on_versions(net, net, w0, X, Y, ver_of, push_seed=773, mu=mu)
    if max(ver_of) > 0:
        assert rel(weights[ver_of.index(1)], weights[ver_of.index(0)]) > 1e-2
    for L in range(lam):
        xs, ys = X[L * mu:(L + 1) * mu], Y[L * mu:(L + 1) * mu]
        rl, rg = cnn.loss_and_gradient(net, weights[L], xs, ys, round_bf16=True)
        # per tensor 2e-2, or 1.5 x the distance between the oracle's own two evaluations of this learner's gradient
        # (reduced-precision and exact) where that is larger: a mini-batch whose ReLU signs sit on bf16 rounding
        # boundaries moves every tensor by a few per cent whichever way the sums are ordered
        _, eg = cnn.loss_and_gradient(net, weights[L], xs, ys)
        _, spread = layer_errors(net, rg, eg)
        _, errs = layer_errors(net, grads[L], rg)
        assert all(e < max(TOL["bf16"], SPREAD_FACTOR * sp) for e, sp in zip(errs, spread)), (L, ver_of, errs, spread)
        if smooth:
            # (with ReLUs a one-ulp difference in a bf16 activation flips hidden units whose input lies within 1e-5 of
            # its terms' magnitude -- every mini-batch here has some -- and a flipped unit moves its whole row of dW)
            ew, at = elem_error(net, grads[L], rg)
            assert ew < ELEM_TOL["bf16"], (L, ver_of, "element", at, ew)
        assert abs(losses[L] - rl) < 2e-2 * max(1.0, abs(rl))


def test_patch_kernel_tiles_spanning_many_small_images():
    # 3 x 3 feature maps: a 128-position tile covers 14 images, each with its own band of halo rows in the patch
    net = wl.tiny_net(3, 5, 5, 6, conv=((32, 3, 1, 0), (64, 3, 1, 1), (96, 2, 1, 1)), pool="avgpool", fc_hidden=16)
    for (g, rg, loss, rl) in one_gradient(net, 40, "bf16", seed=95, lam=2):
        check_gradient(net, "bf16", g, rg, loss, rl, "small images")


@pytest.mark.parametrize("compute", ["fp32", "bf16"])
def test_largest_learner_count_in_one_call(compute):
    """64 learners, the most one context takes, with a mini-batch each in ONE calcGradient call: every learner's
    gradient and loss against the oracle (the pointer tables of a launch are full); 65 learners are refused."""
    from paper_1511_05950_amd import binding
    net = TINY["mfma_pad3"]
    # weights of scale 0.1: at the other tests' 0.3 one of these 64 two-image batches is classified with a loss of 3e-12
    # and its gradient (norm 3e-9) has no meaningful relative error
    seed = decided_seed(net, 64, 2, 164, 0.1) if compute == "fp32" else 164
    for (g, rg, loss, rl) in one_gradient(net, 2, compute, seed=seed, scale=0.1, lam=64):
        check_gradient(net, compute, g, rg, loss, rl, "64 learners")
    theta = np.zeros(wl.num_params(net), dtype=np.float32)
    with pytest.raises(binding.SasgdError):
        binding.Sasgd(65, 2, 65, 2, net=net, compute=compute, init_weights=theta)


@pytest.mark.parametrize("compute", ["fp32", "bf16"])
@pytest.mark.parametrize("name", ["max_clipped", "mfma_pad3", "patch_3x3", "mfma_s4"])
def test_single_image_minibatch(name, compute):
    """mu = 1: the smallest mini-batch (the mean over the mini-batch is the gradient of the one image; every GEMM has
    fewer rows than a tile)."""
    net = TINY[name]
    seed = 7 + sum(map(ord, name))
    if compute == "fp32":
        seed = decided_seed(net, 3, 1, seed, 0.1)
    for (g, rg, loss, rl) in one_gradient(net, 1, compute, seed=seed, scale=0.1, lam=3):
        check_gradient(net, compute, g, rg, loss, rl, name)
