"""Do the oracle's pins bite?  Plausible mistakes are planted in a copy of cnn_oracle.c (on the CPU, never in
the product) and at least one pin -- finite differences or the PyTorch fp64 comparison -- must fail for each."""
import ctypes
import os
import subprocess
import tempfile

import numpy as np
import pytest

import workloads as wl
from oracle import cnn
from test_oracle_cnn import NETS, rand_case, torch_loss

SRC = os.path.join(os.path.dirname(cnn.__file__), "cnn_oracle.c")

MUTATIONS = {
    "conv dx sign": ("dxi[ih * W + iw] += wv * d[oh * OW + ow];", "dxi[ih * W + iw] -= wv * d[oh * OW + ow];"),
    "conv dw transposed window": ("acc += d[oh * OW + ow] * xi[ih * W + iw];", "acc += d[oh * OW + ow] * xi[iw * W + ih];"),
    "conv pad sign": ("int ih = oh * s + kh - p;\n              if (ih < 0 || ih >= H) continue;\n              for (int ow = 0; ow < OW; ow++) {\n                int iw = ow * s + kw - p;\n                if (iw < 0 || iw >= W) continue;\n                yo[",
                      "int ih = oh * s + kh + p;\n              if (ih < 0 || ih >= H) continue;\n              for (int ow = 0; ow < OW; ow++) {\n                int iw = ow * s + kw - p;\n                if (iw < 0 || iw >= W) continue;\n                yo["),
    "bias gradient dropped": ("db[co] = sb;", "db[co] = 0.0;"),
    "no division by mini-batch": ("- (j == label[n] ? 1.0 : 0.0)) / N;", "- (j == label[n] ? 1.0 : 0.0));"),
    "avgpool divides by full window": ("y[((size_t)nc * OH + oh) * OW + ow] = acc / cnt;", "y[((size_t)nc * OH + oh) * OW + ow] = acc / (k * k);"),
    "maxpool last maximum wins": ("if (best < 0 || v > bv)", "if (best < 0 || v >= bv)"),
    "relu backward ignores sign": ("dx[i] = x[i] > 0.0 ? dy[i] : 0.0;", "dx[i] = dy[i];"),
    "fc dx transposed": ("acc += dy[(size_t)n * Out + o] * w[(size_t)o * In + i];", "acc += dy[(size_t)n * Out + o] * w[(size_t)i % Out * In + i];"),
    "pool floor mode": ("int o = (n - k + s - 1) / s + 1;", "int o = (n - k) / s + 1;"),
}


def load_mutant(src_text, tmp):
    c = os.path.join(tmp, "m.c")
    so = os.path.join(tmp, "m.so")
    open(c, "w").write(src_text)
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-shared", "-fPIC", "-o", so, c, "-lm"])
    lib = ctypes.CDLL(so)
    lib.cnn_loss_and_gradient.restype = ctypes.c_double
    return lib


def pins_pass(lib):
    """Finite differences and the torch comparison on the small nets, through the given library."""
    def lg(net, theta, x, y, want=True):
        t = cnn._table(net)
        c, h, w = net["input"]
        theta = np.ascontiguousarray(theta, np.float64)
        x = np.ascontiguousarray(x, np.float64)
        y = np.ascontiguousarray(y, np.int32)
        g = np.empty_like(theta)
        loss = lib.cnn_loss_and_gradient(cnn._dp(t), ctypes.c_int(len(t)), ctypes.c_int(c), ctypes.c_int(h), ctypes.c_int(w),
                                         ctypes.c_int(x.shape[0]), cnn._dp(theta), ctypes.c_long(theta.size), cnn._dp(x), cnn._dp(y),
                                         cnn._dp(g) if want else ctypes.c_void_p(0), ctypes.c_int(0))
        return loss, g
    nets = dict(NETS)
    nets["tie"] = {"name": "t", "input": (2, 3, 3), "classes": 2, "layers": [("conv", 1, 1, 1, 0), ("maxpool", 3, 2), ("fc", 2)]}
    for name, net in nets.items():
        if name == "tie":
            x = np.zeros((1, 2, 3, 3)); x[0, 0, 0, 0] = 2.0; x[0, 1, 2, 2] = 2.0
            theta = np.array([1.0, 1.0, 0.0, 0.7, -0.4, 0.0, 0.0]); y = np.array([0], np.int32)
            _, g = lg(net, theta, x, y)
            if not (g[0] != 0.0 and g[1] == 0.0):
                return False
            continue
        theta, x, y = rand_case(net, 3, 5)
        loss, g = lg(net, theta, x, y)
        if not np.isfinite(loss):
            return False
        tl, tg = torch_loss(net, theta, x, y)
        if abs(loss - tl) > 1e-9 * max(1, abs(tl)) or not np.allclose(g, tg, rtol=1e-8, atol=1e-11):
            return False
        rng = np.random.default_rng(2)
        for k in rng.choice(theta.size, size=12, replace=False):
            tp, tm = theta.copy(), theta.copy()
            tp[k] += 1e-6; tm[k] -= 1e-6
            fd = (lg(net, tp, x, y, False)[0] - lg(net, tm, x, y, False)[0]) / 2e-6
            if abs(fd - g[k]) > 1e-5 * max(1.0, abs(g[k])):
                return False
    return True


def test_unmutated_copy_passes_the_pins():
    with tempfile.TemporaryDirectory() as tmp:
        assert pins_pass(load_mutant(open(SRC).read(), tmp))


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(name):
    old, new = MUTATIONS[name]
    text = open(SRC).read()
    assert text.count(old) >= 1, "mutation target not found: " + name
    with tempfile.TemporaryDirectory() as tmp:
        lib = load_mutant(text.replace(old, new, 1), tmp)
        assert not pins_pass(lib), "no pin noticed: " + name


# ----------------------------------------------------------------------------- protocol engine
import types

import test_oracle_protocol as pins
from oracle import protocol as real_protocol

PROTOCOL_SRC = os.path.join(os.path.dirname(cnn.__file__), "protocol.py")

PROTOCOL_MUTATIONS = {
    "rate ignores staleness": ("return alpha0 / np.maximum(taus, 1).astype(np.float64)", "return np.full(taus.shape, float(alpha0))"),
    "rate off by one": ("np.maximum(taus, 1)", "np.maximum(taus + 1, 1)"),
    "update sign": ("return theta - v_next, v_next", "return theta + v_next, v_next"),
    "no average over c": ("coef = learning_rates(taus, alpha0, mode) / c", "coef = learning_rates(taus, alpha0, mode)"),
    "fresh weights always": ("j = i - tau                             # timestamp", "j = i                                   # timestamp"),
    "momentum dropped": ("v_next = momentum * v + s", "v_next = s"),
    "decay not scaled by rate": ("abar * weight_decay * theta", "weight_decay * theta"),
    "learner order": ("learner = (i * c + l) % lam", "learner = (i + l) % lam"),
    "c rounds up": ("return lam // n", "return -(-lam // n)"),
    "mean staleness uses max": ("max(float(taus.mean()), 1.0)", "max(float(taus.max()), 1.0)"),
}

PIN_TESTS = [getattr(pins, n) for n in dir(pins) if n.startswith("test_") and n != "test_workload_schedules_have_the_stated_shape"]


def run_pins(mod):
    """True if every protocol pin passes with `mod` standing in for oracle.protocol."""
    saved = pins.protocol
    pins.protocol = mod
    try:
        for t in PIN_TESTS:
            marks = [m for m in getattr(t, "pytestmark", []) if m.name == "parametrize"]
            cases = [(v,) if not isinstance(v, (tuple, list)) else tuple(v) for m in marks for v in m.args[1]] or [()]
            for args in cases:
                try:
                    t(*args)
                except Exception:
                    return False
        return True
    finally:
        pins.protocol = saved


def test_protocol_pins_pass_unmutated():
    assert run_pins(real_protocol)


@pytest.mark.parametrize("name", sorted(PROTOCOL_MUTATIONS))
def test_planted_protocol_mistake_is_caught(name):
    old, new = PROTOCOL_MUTATIONS[name]
    text = open(PROTOCOL_SRC).read()
    assert text.count(old) >= 1, "mutation target not found: " + name
    mod = types.ModuleType("mutant_protocol")
    exec(compile(text.replace(old, new, 1), "mutant_protocol", "exec"), mod.__dict__)
    assert not run_pins(mod), "no pin noticed: " + name
