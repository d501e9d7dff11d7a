#!/usr/bin/env python3
"""How far apart are two correct bf16 evaluations of the AlexNet-shaped gradient?  Measured with the CPU oracle alone.

    python tests/golden/make_alex8_bf16_spread.py     # -> tests/golden/alex8_bf16_spread.txt  (about 1 min on 8 cores)

The case is the one the GPU test uses: BASELINE config 4's network and initial weights, one mini-batch of mu = 16
seeded images (seeds 77 / 78).  Three evaluations of calcGradient (Section 2.1):
    E    the oracle's exact mode (float64 throughout);
    R    its reduced-precision mode: tensors between layers rounded to bfloat16, sums in float64;
    R32  the reduced-precision mode of a compiled COPY of cnn_oracle.c in which every running sum of a convolution or
         fully connected layer is rounded to float after each term -- bf16 storage with fp32 accumulation in the
         oracle's loop order, i.e. one more legitimate "bf16 compute" evaluation that differs from R only in how its
         sums round (the copy lives in a temporary directory; the oracle itself is not changed).
Per weight / bias tensor the file lists  ||R - E|| / ||E||,  ||R32 - R|| / ||R||  and  ||R32 - E|| / ||E||.
The GPU kernels are a fourth evaluation of the same kind as R32 (fp32 accumulation in MFMA order); the GPU parity
test bounds its distance to R by twice the R32-to-R spread of the tensor, and its distance to E by twice the R-to-E
spread, wherever those exceed the stated 2e-2.
"""
import ctypes
import os
import subprocess
import sys
import tempfile

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)

import workloads as wl                      # noqa: E402
from oracle import cnn                      # noqa: E402

SRC = os.path.join(os.path.dirname(cnn.__file__), "cnn_oracle.c")

# running sums of the contraction loops, each rounded to float after every term in the copy
FLOAT_SUMS = [
    ("yo[oh * OW + ow] += wv * xi[ih * W + iw];",
     "yo[oh * OW + ow] = (double)((float)yo[oh * OW + ow] + (float)wv * (float)xi[ih * W + iw]);"),
    ("acc += d[oh * OW + ow] * xi[ih * W + iw];",
     "acc = (double)((float)acc + (float)d[oh * OW + ow] * (float)xi[ih * W + iw]);"),
    ("dxi[ih * W + iw] += wv * d[oh * OW + ow];",
     "dxi[ih * W + iw] = (double)((float)dxi[ih * W + iw] + (float)wv * (float)d[oh * OW + ow]);"),
    ("acc += w[(size_t)o * In + i] * x[(size_t)n * In + i];",
     "acc = (double)((float)acc + (float)w[(size_t)o * In + i] * (float)x[(size_t)n * In + i]);"),
    ("acc += dy[(size_t)n * Out + o] * x[(size_t)n * In + i];",
     "acc = (double)((float)acc + (float)dy[(size_t)n * Out + o] * (float)x[(size_t)n * In + i]);"),
    ("acc += dy[(size_t)n * Out + o] * w[(size_t)o * In + i];",
     "acc = (double)((float)acc + (float)dy[(size_t)n * Out + o] * (float)w[(size_t)o * In + i]);"),
    ("for (int i = 0; i < OH * OW; i++) sb += d[i];",
     "for (int i = 0; i < OH * OW; i++) sb = (double)((float)sb + (float)d[i]);"),
    ("for (int n = 0; n < N; n++) sb += dy[(size_t)n * Out + o];",
     "for (int n = 0; n < N; n++) sb = (double)((float)sb + (float)dy[(size_t)n * Out + o]);"),
]


def float_sum_copy(tmp):
    """Compile the copy with float running sums; returns a loss_and_gradient(net, theta, x, label) for its reduced mode."""
    text = open(SRC).read()
    for old, new in FLOAT_SUMS:
        assert text.count(old) == 1, old
        text = text.replace(old, new)
    c, so = os.path.join(tmp, "f32sums.c"), os.path.join(tmp, "f32sums.so")
    open(c, "w").write(text)
    subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-o", so, c, "-lm"])
    lib = ctypes.CDLL(so)
    lib.cnn_loss_and_gradient.restype = ctypes.c_double

    def lg(net, theta, x, label):
        t = cnn._table(net)
        ch, h, w = net["input"]
        theta = np.ascontiguousarray(theta, np.float64)
        x = np.ascontiguousarray(x, np.float64)
        label = np.ascontiguousarray(label, np.int32)
        g = np.empty_like(theta)
        loss = lib.cnn_loss_and_gradient(cnn._dp(t), ctypes.c_int(len(t)), ctypes.c_int(ch), ctypes.c_int(h), ctypes.c_int(w),
                                         ctypes.c_int(x.shape[0]), cnn._dp(theta), ctypes.c_long(theta.size), cnn._dp(x),
                                         cnn._dp(label), cnn._dp(g), ctypes.c_int(1))
        return float(loss), g
    return lg


def tensor_names(net):
    names, k = [], 0
    for L in net["layers"]:
        if L[0] in ("conv", "fc"):
            k += 1
            names += ["%s%d.w" % (L[0], k), "%s%d.b" % (L[0], k)]
    return names


def tensor_ranges(net):
    out, pos = [], 0
    for ws, nb in wl.param_shapes(net):
        nw = int(np.prod(ws))
        out += [(pos, pos + nw), (pos + nw, pos + nw + nb)]
        pos += nw + nb
    return out


def rel(a, b):
    return float(np.linalg.norm(a - b) / np.linalg.norm(b))


def case():
    cfgd = wl.config(4)
    net = cfgd["net"]
    return net, cfgd["weights"](), wl.images(net, cfgd["mu"], 77), wl.labels(net, cfgd["mu"], 78)


def spreads(net, E, R, R32):
    rows = [("whole", rel(R, E), rel(R32, R), rel(R32, E))]
    for name, (a, b) in zip(tensor_names(net), tensor_ranges(net)):
        rows.append((name, rel(R[a:b], E[a:b]), rel(R32[a:b], R[a:b]), rel(R32[a:b], E[a:b])))
    return rows


def main():
    net, w0, X, Y = case()
    lE, E = cnn.loss_and_gradient(net, w0, X, Y)
    lR, R = cnn.loss_and_gradient(net, w0, X, Y, round_bf16=True)
    with tempfile.TemporaryDirectory() as tmp:
        lR32, R32 = float_sum_copy(tmp)(net, w0, X, Y)
    path = os.path.join(HERE, "alex8_bf16_spread.txt")
    with open(path, "w") as f:
        f.write("# Spread between three CPU evaluations of one AlexNet-shaped bf16 gradient (BASELINE config 4, mu = 16, seeds 77/78).\n")
        f.write("# Written by tests/golden/make_alex8_bf16_spread.py from the oracle alone; see that file for E, R, R32.\n")
        f.write("# loss E %.12g   loss R %.12g   loss R32 %.12g\n" % (lE, lR, lR32))
        f.write("# tensor        |R-E|/|E|     |R32-R|/|R|   |R32-E|/|E|\n")
        for (name, a, b, c) in spreads(net, E, R, R32):
            f.write("%-12s  %.4e   %.4e   %.4e\n" % (name, a, b, c))
    print(open(path).read())


if __name__ == "__main__":
    main()
