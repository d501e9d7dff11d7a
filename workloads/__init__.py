"""Seeded synthetic workloads for staleness-aware n-softsync ASGD.

This module serves the CPU oracle's tests, the GPU parity tests and bench.py alike.
It holds shapes, hyper-parameters and random draws only -- none of the method's
arithmetic (no gradient, no update rule, no learning-rate formula).  Random numbers
come from numpy's default_rng with fixed seeds, so both sides see identical inputs.

Network descriptions are plain tuples:
    ("conv", cout, k, stride, pad)   square k x k convolution with bias
    ("maxpool", k, stride)           ceil-mode window, clipped at the border
    ("avgpool", k, stride)           same geometry, mean over in-bounds elements
    ("relu",)
    ("fc", out)                      fully connected with bias (input flattened C,H,W)
The loss (softmax cross-entropy, mean over the mini-batch) is implied after the last layer.

The two networks stand in for the CIFAR10 and ImageNet models of the paper's Section 4.1;
the datasets themselves are replaced by N(0,1) pixels and uniform labels of the same shapes.
"""
from __future__ import annotations

import numpy as np

SEED0 = 15110595


# --------------------------------------------------------------------------- networks
CIFAR3 = {
    "name": "cifar3",
    "input": (3, 32, 32),
    "classes": 10,
    "layers": [
        ("conv", 32, 5, 1, 2), ("maxpool", 3, 2), ("relu",),
        ("conv", 32, 5, 1, 2), ("relu",), ("avgpool", 3, 2),
        ("conv", 64, 5, 1, 2), ("relu",), ("avgpool", 3, 2),
        ("fc", 10),
    ],
}

ALEX8 = {
    "name": "alex8",
    "input": (3, 224, 224),
    "classes": 1000,
    "layers": [
        ("conv", 96, 11, 4, 0), ("relu",), ("maxpool", 3, 2),
        ("conv", 256, 5, 1, 2), ("relu",), ("maxpool", 3, 2),
        ("conv", 384, 3, 1, 1), ("relu",),
        ("conv", 384, 3, 1, 1), ("relu",),
        ("conv", 256, 3, 1, 1), ("relu",), ("maxpool", 3, 2),
        ("fc", 4096), ("relu",),
        ("fc", 4096), ("relu",),
        ("fc", 1000),
    ],
}


# Same layer shapes as ALEX8 with every decision removed (no ReLU, average instead of max pooling): the loss is a
# smooth function of the parameters, so reduced-precision runs can be compared at a tight tolerance at full size.
ALEX8_SMOOTH = {
    "name": "alex8_smooth",
    "input": (3, 224, 224),
    "classes": 1000,
    "layers": [("avgpool", L[1], L[2]) if L[0] == "maxpool" else L for L in ALEX8["layers"] if L[0] != "relu"],
}


def tiny_net(c=3, h=9, w=7, classes=5, conv=((4, 3, 1, 1),), pool="maxpool", fc_hidden=None):
    """A small net for gradient checks: conv(s) -> pool -> relu -> [fc relu] -> fc."""
    layers = []
    for (co, k, s, p) in conv:
        layers += [("conv", co, k, s, p), ("relu",)]
    layers += [(pool, 3, 2)]
    if fc_hidden:
        layers += [("fc", fc_hidden), ("relu",)]
    layers += [("fc", classes)]
    return {"name": "tiny", "input": (c, h, w), "classes": classes, "layers": layers}


def _pool_out(n, k, s):
    # ceil-mode output size; every window starts inside the input
    o = -(-(n - k) // s) + 1
    if (o - 1) * s >= n:
        o -= 1
    return max(o, 1)


def param_shapes(net):
    """[(weight_shape, bias_len)] for every conv/fc layer, in network order."""
    c, h, w = net["input"]
    out = []
    for L in net["layers"]:
        if L[0] == "conv":
            _, co, k, s, p = L
            out.append(((co, c, k, k), co))
            h = (h + 2 * p - k) // s + 1
            w = (w + 2 * p - k) // s + 1
            c = co
        elif L[0] in ("maxpool", "avgpool"):
            _, k, s = L
            h, w = _pool_out(h, k, s), _pool_out(w, k, s)
        elif L[0] == "fc":
            out.append(((L[1], c * h * w), L[1]))
            c, h, w = L[1], 1, 1
    return out


def num_params(net):
    return sum(int(np.prod(ws)) + b for ws, b in param_shapes(net))


# --------------------------------------------------------------------------- draws
def init_weights(net, seed, std=0.01):
    """Flat fp32 parameter vector: per layer Gaussian(0, std) weights then zero biases."""
    rng = np.random.default_rng(seed)
    parts = []
    for ws, b in param_shapes(net):
        parts.append((rng.standard_normal(int(np.prod(ws))) * std).astype(np.float32))
        parts.append(np.zeros(b, np.float32))
    return np.concatenate(parts)


def images(net, count, seed):
    c, h, w = net["input"]
    return np.random.default_rng(seed).standard_normal((count, c, h, w), dtype=np.float32)


def labels(net, count, seed):
    return np.random.default_rng(seed).integers(0, net["classes"], size=count, dtype=np.int32)


def uniform_schedule(K, c, lo, hi, seed):
    """int32[K][c], each entry uniform in {lo..hi} (inclusive)."""
    return np.random.default_rng(seed).integers(lo, hi + 1, size=(K, c), dtype=np.int32)


def jitter_schedule(K, c, n, seed):
    """Round-robin-with-jitter: n + J clipped to [0, 2n], J uniform integer in [-n/2, n/2].

    Mimics the measured staleness shape for n-softsync (Section 2.4, Figure 1): the mass
    sits near n and stays within 2n.
    """
    j = np.random.default_rng(seed).integers(-(n // 2), n // 2 + 1, size=(K, c))
    return np.clip(n + j, 0, 2 * n).astype(np.int32)


# --------------------------------------------------------------------------- configs
def _cfg_seed(cfg, k=0):
    return SEED0 + 1000 * cfg + k


def config(cfg):
    """Hyper-parameters and generators of BASELINE config `cfg` (0..4)."""
    if cfg == 0:
        d = dict(net=CIFAR3, compute="fp32", lam=4, mu=4, n=1, K=8, alpha0=1e-3, momentum=0.9,
                 weight_decay=0.0, lr_mode="per_gradient")
        d["schedule"] = lambda: uniform_schedule(8, 4, 0, 4, _cfg_seed(0, 3))
    elif cfg == 1:
        d = dict(net=None, compute="fp32", lam=54, mu=0, n=54, K=54, alpha0=1e-2, momentum=0.9,
                 weight_decay=5e-4, lr_mode="per_gradient", num_params=60_000_000,
                 grad_std=1e-3)
        d["staleness"] = lambda: np.random.default_rng(_cfg_seed(1, 3)).integers(
            0, 2 * 54 + 1, size=54, dtype=np.int32)
    elif cfg == 2:
        d = dict(net=CIFAR3, compute="fp32", lam=30, mu=4, n=30, K=200, alpha0=1e-3, momentum=0.9,
                 weight_decay=0.0, lr_mode="per_gradient")
        d["schedule"] = lambda: jitter_schedule(200, 1, 30, _cfg_seed(2, 3))
    elif cfg == 3:
        d = dict(net=CIFAR3, compute="bf16", lam=18, mu=128, n=1, K=100, alpha0=1e-3, momentum=0.9,
                 weight_decay=0.0, lr_mode="per_gradient", image_pool=2304)
        d["schedule"] = lambda: uniform_schedule(100, 18, 0, 2, _cfg_seed(3, 3))
    elif cfg == 4:
        d = dict(net=ALEX8, compute="bf16", lam=18, mu=16, n=18, K=20, alpha0=1e-2, momentum=0.9,
                 weight_decay=5e-4, lr_mode="per_gradient")
        d["schedule"] = lambda: uniform_schedule(20, 1, 0, 36, _cfg_seed(4, 3))
    else:
        raise ValueError(cfg)
    d["cfg"] = cfg
    d["c"] = d["lam"] // d["n"]
    if d["net"] is not None:
        net = d["net"]
        n_img = d.get("image_pool", d["K"] * d["c"] * d["mu"])
        d["n_images"] = n_img
        d["images"] = lambda: images(net, n_img, _cfg_seed(cfg, 0))
        d["labels"] = lambda: labels(net, n_img, _cfg_seed(cfg, 1))
        d["weights"] = lambda: init_weights(net, _cfg_seed(cfg, 2))
    return d


def batch_slice(cfgd, i, l):
    """Index range into the image/label arrays of the l-th gradient of update i."""
    g = i * cfgd["c"] + l
    mu = cfgd["mu"]
    start = (g * mu) % cfgd["n_images"]
    return slice(start, start + mu)


def server_vector(P, seed, std):
    """fp32 Gaussian vector of length P generated in bounded chunks."""
    rng = np.random.default_rng(seed)
    out = np.empty(P, np.float32)
    step = 1 << 22
    for s in range(0, P, step):
        e = min(P, s + step)
        out[s:e] = rng.standard_normal(e - s, dtype=np.float32) * np.float32(std)
    return out


def config1_theta(P=60_000_000):
    return server_vector(P, _cfg_seed(1, 2), 0.01)


def config1_gradient(l, P=60_000_000):
    return server_vector(P, _cfg_seed(1, 4 + l), 1e-3)
