"""ctypes binding of libsasgd.so: argument marshalling only, same names as the C ABI (include/sasgd.h).

Device buffers are passed as torch CUDA tensors (their data_ptr is forwarded) or raw integer addresses.
The library is required: there is no fallback path, loading fails loudly when it has not been built.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsasgd.so")

OK, EINVAL, ESTATE, ENOTREADY, ERANGE, EHIP, ENOMEM = 0, -1, -2, -3, -4, -5, -6
NET_NONE, NET_CIFAR3, NET_ALEX8, NET_CUSTOM = 0, 1, 2, 3
FP32, BF16 = 0, 1
LR_PER_GRADIENT, LR_MEAN_STALENESS, LR_CONSTANT = 0, 1, 2
LAYER_KINDS = {"conv": 0, "maxpool": 1, "avgpool": 2, "relu": 3, "fc": 4}
LR_MODES = {"per_gradient": 0, "mean_staleness": 1, "constant": 2}
FLAG_FLAT_FC_GRADIENT = 1
FLAG_EAGER_UPDATES = 2
COMPUTE = {"fp32": 0, "bf16": 1}

EXPORTS = [
    "sasgd_create", "sasgd_destroy", "sasgd_getMinibatch", "sasgd_pullWeights", "sasgd_calcGradient",
    "sasgd_pushGradient", "sasgd_pushGradientExternal", "sasgd_sumGradients", "sasgd_applyUpdate",
    "sasgd_timestamp", "sasgd_numParams", "sasgd_gradientsPerUpdate", "sasgd_gradientTimestamp",
    "sasgd_copyWeights", "sasgd_copyGradient", "sasgd_copyMomentum", "sasgd_gradientPtr",
    "sasgd_setProfiling", "sasgd_phaseTime", "sasgd_last_error", "sasgd_version",
    "sasgd_evaluate", "sasgd_setBaseRate", "sasgd_setPixelMean", "sasgd_factoredParams",
    "sasgd_applyUpdateNoAlloc", "sasgd_flush",
]


class SasgdLayer(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("units", ctypes.c_int32), ("window", ctypes.c_int32),
                ("stride", ctypes.c_int32), ("pad", ctypes.c_int32)]


ALLOC_FN = ctypes.CFUNCTYPE(ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p)
RELEASE_FN = ctypes.CFUNCTYPE(None, ctypes.c_void_p, ctypes.c_void_p)


class SasgdConfig(ctypes.Structure):
    _fields_ = [
        ("lambda_", ctypes.c_int32), ("mu", ctypes.c_int32), ("n", ctypes.c_int32), ("ring_depth", ctypes.c_int32),
        ("net", ctypes.c_int32), ("compute", ctypes.c_int32), ("lr_mode", ctypes.c_int32), ("flags", ctypes.c_int32),
        ("num_params", ctypes.c_int64),
        ("alpha0", ctypes.c_float), ("momentum", ctypes.c_float), ("weight_decay", ctypes.c_float), ("reserved1", ctypes.c_float),
        ("stream", ctypes.c_void_p),
        ("layers", ctypes.POINTER(SasgdLayer)), ("num_layers", ctypes.c_int32),
        ("in_channels", ctypes.c_int32), ("in_height", ctypes.c_int32), ("in_width", ctypes.c_int32),
        ("alloc", ALLOC_FN), ("release", RELEASE_FN), ("alloc_user", ctypes.c_void_p),
    ]


class SasgdError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("sasgd error %d: %s" % (code, msg))
        self.code = code


_lib = None


def load():
    """Load libsasgd.so (built by paper_1511_05950_amd.build); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                LIB_PATH + " is missing: build it with `python -m paper_1511_05950_amd.build` (no CPU fallback exists)")
        lib = ctypes.CDLL(LIB_PATH)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        P = ctypes.POINTER
        lib.sasgd_create.argtypes = [P(SasgdConfig), vp, P(vp)]
        lib.sasgd_destroy.argtypes = [vp]
        lib.sasgd_getMinibatch.argtypes = [vp, i32, vp, vp]
        lib.sasgd_pullWeights.argtypes = [vp, i32, i32, P(i64)]
        lib.sasgd_calcGradient.argtypes = [vp, P(i32), i32, vp]
        lib.sasgd_pushGradient.argtypes = [vp, i32, P(i32)]
        lib.sasgd_pushGradientExternal.argtypes = [vp, vp, i64, P(i32)]
        lib.sasgd_sumGradients.argtypes = [vp, P(i32)]
        lib.sasgd_applyUpdate.argtypes = [vp, P(i64)]
        lib.sasgd_flush.argtypes = [vp]
        lib.sasgd_timestamp.argtypes = [vp, P(i64)]
        lib.sasgd_numParams.argtypes = [vp, P(i64)]
        lib.sasgd_gradientsPerUpdate.argtypes = [vp, P(i32)]
        lib.sasgd_factoredParams.argtypes = [vp, P(i64)]
        lib.sasgd_gradientTimestamp.argtypes = [vp, i32, P(i64)]
        lib.sasgd_copyWeights.argtypes = [vp, i64, vp]
        lib.sasgd_copyGradient.argtypes = [vp, i32, vp]
        lib.sasgd_copyMomentum.argtypes = [vp, vp]
        lib.sasgd_gradientPtr.argtypes = [vp, i32, P(vp)]
        lib.sasgd_setProfiling.argtypes = [vp, i32]
        lib.sasgd_phaseTime.argtypes = [vp, i32, P(ctypes.c_double), P(i64)]
        lib.sasgd_evaluate.argtypes = [vp, P(i32), i32, vp, vp]
        lib.sasgd_setBaseRate.argtypes = [vp, ctypes.c_float]
        lib.sasgd_setPixelMean.argtypes = [vp, vp]
        lib.sasgd_applyUpdateNoAlloc.argtypes = [vp, vp, vp, vp, i64, i32, P(vp), P(i32), i32, ctypes.c_float, ctypes.c_float,
                                                 ctypes.c_float, vp, ctypes.c_char_p, ctypes.c_size_t]
        lib.sasgd_last_error.argtypes = [vp]
        lib.sasgd_last_error.restype = ctypes.c_char_p
        lib.sasgd_version.restype = ctypes.c_char_p
        for name in EXPORTS:
            if name not in ("sasgd_last_error", "sasgd_version"):
                getattr(lib, name).restype = ctypes.c_int
        _lib = lib
    return _lib


def _addr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):          # torch tensor
        return x.data_ptr()
    if isinstance(x, np.ndarray):
        return x.ctypes.data
    raise TypeError(type(x))


class Sasgd:
    """One context of the C library.  Methods mirror the C calls one to one."""

    def __init__(self, lam, mu, n, ring_depth, net=None, compute="fp32", lr_mode="per_gradient",
                 num_params=0, alpha0=0.01, momentum=0.0, weight_decay=0.0, init_weights=None, stream=None, flags=0):
        lib = load()
        cfg = SasgdConfig()
        cfg.lambda_, cfg.mu, cfg.n, cfg.ring_depth = lam, mu, n, ring_depth
        cfg.compute = COMPUTE[compute] if isinstance(compute, str) else compute
        cfg.lr_mode = LR_MODES[lr_mode] if isinstance(lr_mode, str) else lr_mode
        cfg.num_params = num_params
        cfg.flags = flags
        cfg.alpha0, cfg.momentum, cfg.weight_decay = alpha0, momentum, weight_decay
        if stream is None:
            import torch
            stream = torch.cuda.current_stream().cuda_stream
        cfg.stream = stream
        self._layers = None
        if net is None:
            cfg.net = NET_NONE
        elif net in ("cifar3", NET_CIFAR3):
            cfg.net = NET_CIFAR3
        elif net in ("alex8", NET_ALEX8):
            cfg.net = NET_ALEX8
        else:                               # dict(input=(C,H,W), layers=[tuples])
            cfg.net = NET_CUSTOM
            rows = net["layers"]
            arr = (SasgdLayer * len(rows))()
            for k, L in enumerate(rows):
                vals = list(L[1:]) + [0] * 4
                arr[k].kind = LAYER_KINDS[L[0]]
                if L[0] == "conv":
                    arr[k].units, arr[k].window, arr[k].stride, arr[k].pad = vals[:4]
                elif L[0] in ("maxpool", "avgpool"):
                    arr[k].window, arr[k].stride = vals[:2]
                elif L[0] == "fc":
                    arr[k].units = vals[0]
            self._layers = arr
            cfg.layers = arr
            cfg.num_layers = len(rows)
            cfg.in_channels, cfg.in_height, cfg.in_width = net["input"]
        self._cfg = cfg
        self._h = ctypes.c_void_p()
        w = init_weights
        if isinstance(w, np.ndarray):
            w = np.ascontiguousarray(w, dtype=np.float32)
        self._keep = w
        rc = lib.sasgd_create(ctypes.byref(cfg), _addr(w), ctypes.byref(self._h))
        if rc != OK:
            self._h = ctypes.c_void_p()
            raise SasgdError(rc, "sasgd_create failed (see stderr)")
        self._keep = None
        self.P = self.numParams()
        self.c = self.gradientsPerUpdate()

    # -- plumbing
    def _check(self, rc):
        if rc != OK:
            raise SasgdError(rc, load().sasgd_last_error(self._h).decode())
        return rc

    def destroy(self):
        if self._h:
            load().sasgd_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    # -- learner side
    def getMinibatch(self, learner, images_dev, labels_dev):
        self._check(load().sasgd_getMinibatch(self._h, learner, _addr(images_dev), _addr(labels_dev)))

    def pullWeights(self, learner, staleness_request=0):
        ts = ctypes.c_int64()
        self._check(load().sasgd_pullWeights(self._h, learner, staleness_request, ctypes.byref(ts)))
        return ts.value

    def calcGradient(self, learners, out_loss_dev=None):
        arr = (ctypes.c_int32 * len(learners))(*learners)
        self._check(load().sasgd_calcGradient(self._h, arr, len(learners), _addr(out_loss_dev)))

    def pushGradient(self, learner):
        tau = ctypes.c_int32()
        self._check(load().sasgd_pushGradient(self._h, learner, ctypes.byref(tau)))
        return tau.value

    def pushGradientExternal(self, grad_dev, timestamp):
        tau = ctypes.c_int32()
        self._check(load().sasgd_pushGradientExternal(self._h, _addr(grad_dev), timestamp, ctypes.byref(tau)))
        return tau.value

    # -- training-loop pieces around the hot path
    def evaluate(self, learners, out_loss_dev, out_rank_dev):
        arr = (ctypes.c_int32 * len(learners))(*learners)
        self._check(load().sasgd_evaluate(self._h, arr, len(learners), _addr(out_loss_dev), _addr(out_rank_dev)))

    def setBaseRate(self, alpha0):
        self._check(load().sasgd_setBaseRate(self._h, alpha0))

    def setPixelMean(self, mean_dev):
        self._keep_mean = mean_dev          # the library reads it on every later calcGradient / evaluate
        self._check(load().sasgd_setPixelMean(self._h, _addr(mean_dev)))

    # -- server side
    def sumGradients(self):
        pending = ctypes.c_int32()
        self._check(load().sasgd_sumGradients(self._h, ctypes.byref(pending)))
        return pending.value

    def applyUpdate(self):
        ts = ctypes.c_int64()
        self._check(load().sasgd_applyUpdate(self._h, ctypes.byref(ts)))
        return ts.value

    def flush(self):
        self._check(load().sasgd_flush(self._h))

    # -- getters
    def timestamp(self):
        ts = ctypes.c_int64()
        self._check(load().sasgd_timestamp(self._h, ctypes.byref(ts)))
        return ts.value

    def numParams(self):
        p = ctypes.c_int64()
        self._check(load().sasgd_numParams(self._h, ctypes.byref(p)))
        return p.value

    def gradientsPerUpdate(self):
        c = ctypes.c_int32()
        self._check(load().sasgd_gradientsPerUpdate(self._h, ctypes.byref(c)))
        return c.value

    def factoredParams(self):
        n = ctypes.c_int64()
        self._check(load().sasgd_factoredParams(self._h, ctypes.byref(n)))
        return n.value

    def gradientTimestamp(self, learner):
        ts = ctypes.c_int64()
        self._check(load().sasgd_gradientTimestamp(self._h, learner, ctypes.byref(ts)))
        return ts.value

    def copyWeights(self, version=None):
        out = np.empty(self.P, np.float32)
        self._check(load().sasgd_copyWeights(self._h, self.timestamp() if version is None else version, _addr(out)))
        return out

    def copyGradient(self, learner):
        out = np.empty(self.P, np.float32)
        self._check(load().sasgd_copyGradient(self._h, learner, _addr(out)))
        return out

    def copyMomentum(self):
        out = np.empty(self.P, np.float32)
        self._check(load().sasgd_copyMomentum(self._h, _addr(out)))
        return out

    def gradientPtr(self, learner):
        p = ctypes.c_void_p()
        self._check(load().sasgd_gradientPtr(self._h, learner, ctypes.byref(p)))
        return p.value

    def setProfiling(self, on):
        self._check(load().sasgd_setProfiling(self._h, 1 if on else 0))

    def phaseTime(self, which):
        ms, calls = ctypes.c_double(), ctypes.c_int64()
        self._check(load().sasgd_phaseTime(self._h, which, ctypes.byref(ms), ctypes.byref(calls)))
        return ms.value, calls.value

    def last_error(self):
        return load().sasgd_last_error(self._h).decode()


def applyUpdateNoAlloc(theta_in_dev, theta_out_dev, v_dev, grads_dev, staleness, lr_mode="per_gradient", alpha0=0.01,
                       momentum=0.0, weight_decay=0.0, shadow_out_dev=None, num_params=None, stream=None):
    """sasgd_applyUpdateNoAlloc: the context-free server update that allocates nothing (see include/sasgd.h).
    grads_dev: sequence of device tensors / addresses; staleness: sequence of ints."""
    lib = load()
    c = len(grads_dev)
    if num_params is None:
        num_params = int(theta_in_dev.numel())
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    ptrs = (ctypes.c_void_p * max(c, 1))(*[_addr(g) for g in grads_dev])
    taus = (ctypes.c_int32 * max(c, 1))(*[int(t) for t in staleness])
    err = ctypes.create_string_buffer(256)
    rc = lib.sasgd_applyUpdateNoAlloc(_addr(theta_in_dev), _addr(theta_out_dev), _addr(v_dev), _addr(shadow_out_dev), num_params, c,
                                      ptrs, taus, LR_MODES[lr_mode] if isinstance(lr_mode, str) else lr_mode, alpha0, momentum,
                                      weight_decay, stream, err, len(err))
    if rc != OK:
        raise SasgdError(rc, err.value.decode())
    return rc


def version():
    return load().sasgd_version().decode()
