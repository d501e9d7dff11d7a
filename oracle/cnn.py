"""ctypes front end of cnn_oracle.c (test infrastructure; see that file's header).

calcGradient (Section 2.1): the gradient of the mini-batch loss divided by the
mini-batch size, for the layer types of Section 4.1.  Everything is float64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cnn_oracle.c")
_LIB = os.path.join(_HERE, "libcnn_oracle.so")
_lib = None

_TYPES = {"conv": 0, "maxpool": 1, "avgpool": 2, "relu": 3, "fc": 4}


def build(force=False):
    """Compile cnn_oracle.c with gcc (-O2, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.cnn_loss_and_gradient.restype = ctypes.c_double
        _lib.cnn_class_scores.restype = ctypes.c_double
        _lib.cnn_num_params.restype = ctypes.c_long
        _lib.cnn_min_relu_margin.restype = ctypes.c_double
        _lib.round_to_bf16.restype = ctypes.c_double
        _lib.round_to_bf16.argtypes = [ctypes.c_double]
    return _lib


def _table(net):
    rows = []
    for L in net["layers"]:
        vals = list(L[1:]) + [0] * (5 - len(L))
        rows.append([_TYPES[L[0]]] + vals[:4])
    return np.ascontiguousarray(rows, dtype=np.int32)


def _dp(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def num_params(net):
    t = _table(net)
    c, h, w = net["input"]
    return int(lib().cnn_num_params(_dp(t), ctypes.c_int(len(t)), ctypes.c_int(c), ctypes.c_int(h), ctypes.c_int(w)))


def round_to_bf16(v):
    """Nearest bfloat16 (ties to even) of a float."""
    return float(lib().round_to_bf16(float(v)))


def loss_and_gradient(net, theta, x, label, want_grad=True, round_bf16=False):
    """(loss, grad) of one mini-batch; grad is the mean over the mini-batch (None if not wanted).

    round_bf16: reduced-precision mode, tensors held between layers are rounded to bfloat16
    (see cnn_oracle.c)."""
    t = _table(net)
    c, h, w = net["input"]
    theta = np.ascontiguousarray(theta, dtype=np.float64)
    x = np.ascontiguousarray(x, dtype=np.float64)
    label = np.ascontiguousarray(label, dtype=np.int32)
    n = x.shape[0]
    assert x.shape == (n, c, h, w) and label.shape == (n,)
    assert label.min() >= 0 and label.max() < net["classes"]
    grad = np.empty_like(theta) if want_grad else None
    loss = lib().cnn_loss_and_gradient(
        _dp(t), ctypes.c_int(len(t)), ctypes.c_int(c), ctypes.c_int(h), ctypes.c_int(w), ctypes.c_int(n),
        _dp(theta), ctypes.c_long(theta.size), _dp(x), _dp(label),
        _dp(grad) if want_grad else ctypes.c_void_p(0), ctypes.c_int(1 if round_bf16 else 0))
    if not np.isfinite(loss) and np.isnan(loss):
        raise ValueError("parameter vector length does not match the network")
    return float(loss), grad


def min_relu_margin(net, theta, x):
    """Smallest |v| / sum|terms| over every ReLU input v of this case (exact mode; see cnn_oracle.c).  Below about
    1e-6 some ReLU input is smaller than the rounding error of a float sum of its terms, so its sign, and with it
    the gradient, is not defined at fp32 precision."""
    t = _table(net)
    c, h, w = net["input"]
    theta = np.ascontiguousarray(theta, dtype=np.float64)
    x = np.ascontiguousarray(x, dtype=np.float64)
    m = lib().cnn_min_relu_margin(_dp(t), ctypes.c_int(len(t)), ctypes.c_int(c), ctypes.c_int(h), ctypes.c_int(w),
                                  ctypes.c_int(x.shape[0]), _dp(theta), ctypes.c_long(theta.size), _dp(x))
    if np.isnan(m):
        raise ValueError("parameter vector length does not match the network")
    return float(m)


def make_callback(net, round_bf16=False):
    """grad(theta, (x, label)) -> (g, loss) for oracle.protocol.run."""
    def cb(theta, batch):
        loss, g = loss_and_gradient(net, theta, batch[0], batch[1], round_bf16=round_bf16)
        return g, loss
    return cb


def class_scores(net, theta, x, label, round_bf16=False):
    """(loss, scores[N][classes]) of a forward-only evaluation pass (Section 4.3: test / validation error)."""
    t = _table(net)
    c, h, w = net["input"]
    theta = np.ascontiguousarray(theta, dtype=np.float64)
    x = np.ascontiguousarray(x, dtype=np.float64)
    label = np.ascontiguousarray(label, dtype=np.int32)
    n = x.shape[0]
    assert x.shape == (n, c, h, w) and label.shape == (n,)
    scores = np.empty((n, net["classes"]), np.float64)
    loss = lib().cnn_class_scores(
        _dp(t), ctypes.c_int(len(t)), ctypes.c_int(c), ctypes.c_int(h), ctypes.c_int(w), ctypes.c_int(n),
        _dp(theta), ctypes.c_long(theta.size), _dp(x), _dp(label), _dp(scores), ctypes.c_int(1 if round_bf16 else 0))
    return float(loss), scores


def label_rank(scores, label):
    """Position of the true class when the classes are sorted by descending score (equal scores: lower index
    first).  rank >= 1 is a top-1 error, rank >= 5 a top-5 error (the error measures of Section 4.3)."""
    scores = np.asarray(scores)
    out = np.empty(len(label), np.int32)
    for s in range(len(label)):
        y = int(label[s])
        zy = scores[s, y]
        before = 0
        for j in range(scores.shape[1]):
            if scores[s, j] > zy or (scores[s, j] == zy and j < y):
                before += 1
        out[s] = before
    return out
