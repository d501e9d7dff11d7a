"""Pins for the oracle's training-loop pieces around the hot path: evaluation pass (class scores, rank of the
true class), step decay of the base rate (Sections 4.1 - 4.3).  None of them re-types the oracle's code."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workloads as wl
from oracle import cnn, protocol

from test_oracle_cnn import NETS, gold, rand_case
from test_oracle_protocol import lsq_callback, lsq_problem


def torch_scores(net, theta, x):
    t = torch.tensor(theta, dtype=torch.float64)
    a = torch.tensor(x, dtype=torch.float64)
    pos = 0
    for L in net["layers"]:
        if L[0] == "conv":
            _, co, k, s, p = L
            nw = co * a.shape[1] * k * k
            a = F.conv2d(a, t[pos:pos + nw].reshape(co, a.shape[1], k, k), t[pos + nw:pos + nw + co], stride=s, padding=p)
            pos += nw + co
        elif L[0] == "maxpool":
            a = F.max_pool2d(a, L[1], L[2], ceil_mode=True)
        elif L[0] == "avgpool":
            a = F.avg_pool2d(a, L[1], L[2], ceil_mode=True, count_include_pad=False)
        elif L[0] == "relu":
            a = F.relu(a)
        elif L[0] == "fc":
            a = a.reshape(a.shape[0], -1)
            nw = L[1] * a.shape[1]
            a = F.linear(a, t[pos:pos + nw].reshape(L[1], a.shape[1]), t[pos + nw:pos + nw + L[1]])
            pos += nw + L[1]
    return a.reshape(a.shape[0], -1).numpy()


@pytest.mark.parametrize("name", ["max_clipped", "stride2_pad", "cifar3"])
def test_class_scores_against_torch_forward(name):
    net = wl.CIFAR3 if name == "cifar3" else NETS[name]
    theta, x, y = rand_case(net, 3, 11)
    if name == "cifar3":
        theta = theta * 0.2
    loss, scores = cnn.class_scores(net, theta, x, y)
    ref = torch_scores(net, theta, x)
    np.testing.assert_allclose(scores, ref, rtol=1e-10, atol=1e-11)
    # the loss of the evaluation pass is the training loss of the same batch
    ref_loss = F.cross_entropy(torch.tensor(ref), torch.tensor(y, dtype=torch.long)).item()
    assert abs(loss - ref_loss) < 1e-11 * max(1.0, abs(ref_loss))
    assert loss == cnn.loss_and_gradient(net, theta, x, y, want_grad=False)[0]


def test_label_rank_is_position_in_stable_descending_sort():
    rng = np.random.default_rng(5)
    scores = rng.standard_normal((40, 17))
    scores[:, 3] = scores[:, 9]            # ties between classes 3 and 9 in every row
    label = rng.integers(0, 17, 40).astype(np.int32)
    label[:6] = [3, 9, 3, 9, 0, 16]
    rank = cnn.label_rank(scores, label)
    order = np.argsort(-scores, axis=1, kind="stable")      # equal scores keep the lower class index first
    expect = np.array([int(np.where(order[s] == label[s])[0][0]) for s in range(40)])
    np.testing.assert_array_equal(rank, expect)
    # hand example: scores (1, 5, 5, 0); class 1 wins the tie against class 2
    z = np.array([[1.0, 5.0, 5.0, 0.0]] * 4)
    np.testing.assert_array_equal(cnn.label_rank(z, np.array([0, 1, 2, 3], np.int32)), [2, 0, 1, 3])
    # top-1 / top-5 error counts agree with torch.topk on tie-free scores
    scores = rng.standard_normal((50, 30))
    label = rng.integers(0, 30, 50).astype(np.int32)
    rank = cnn.label_rank(scores, label)
    top5 = torch.topk(torch.tensor(scores), 5, dim=1).indices.numpy()
    assert int((rank >= 5).sum()) == int(sum(label[s] not in top5[s] for s in range(50)))
    assert int((rank >= 1).sum()) == int((scores.argmax(1) != label).sum())


def test_step_decay_reproduces_the_schedules_the_paper_states():
    g = gold()
    per_epoch = 7                           # updates per epoch: any value, the boundaries scale with it
    K = 140 * per_epoch
    a = protocol.step_decay(g["cifar_alpha0"], [int(g["cifar_decay_epoch_a"]) * per_epoch, int(g["cifar_decay_epoch_b"]) * per_epoch],
                            g["cifar_decay_factor"], K)
    assert a[0] == 1e-3 and a[120 * per_epoch - 1] == 1e-3
    np.testing.assert_allclose(a[120 * per_epoch], 1e-4, rtol=1e-15)
    np.testing.assert_allclose(a[130 * per_epoch - 1], 1e-4, rtol=1e-15)
    np.testing.assert_allclose(a[130 * per_epoch:], 1e-5, rtol=1e-15)
    b = protocol.step_decay(g["imagenet_alpha0"], [int(g["imagenet_decay_epoch_a"]), int(g["imagenet_decay_epoch_b"])],
                            g["imagenet_decay_factor"], 35)
    np.testing.assert_allclose(b[[0, 19, 20, 29, 30, 34]], [0.01, 0.01, 0.002, 0.002, 0.0004, 0.0004], rtol=1e-15)


def test_per_update_base_rate_closed_form_and_chaining():
    # no staleness, no momentum: theta_K - theta* = prod_i (I - a_i A) (theta_0 - theta*)
    A, b = lsq_problem(5, 30, 2)
    th0 = np.linspace(-1, 1, 5)
    K = 12
    rates = protocol.step_decay(0.3, [5, 9], 4.0, K)
    out = protocol.run(lsq_callback(A, b), th0, lambda i, l: None, np.zeros((K, 1), int), 3, 3, rates)
    star = np.linalg.solve(A, b)
    M = np.eye(5)
    for i in range(K):
        M = (np.eye(5) - rates[i] * A) @ M
    np.testing.assert_allclose(out["theta"], star + M @ (th0 - star), rtol=1e-11, atol=1e-13)
    # with staleness and momentum: an array of equal rates is the scalar run
    sched = np.random.default_rng(0).integers(0, 4, (K, 2))
    r1 = protocol.run(lsq_callback(A, b), th0, lambda i, l: None, sched, 4, 2, 0.1, momentum=0.8, weight_decay=1e-2)
    r2 = protocol.run(lsq_callback(A, b), th0, lambda i, l: None, sched, 4, 2, np.full(K, 0.1), momentum=0.8, weight_decay=1e-2)
    np.testing.assert_array_equal(r1["theta"], r2["theta"])
    # and the rate of update i scales exactly that update's step (m = wd = 0): halving a_3 halves theta_4 - theta_3
    ra = np.full(K, 0.1)
    rb = ra.copy()
    rb[3] = 0.05
    oa = protocol.run(lsq_callback(A, b), th0, lambda i, l: None, sched, 4, 2, ra)
    ob = protocol.run(lsq_callback(A, b), th0, lambda i, l: None, sched, 4, 2, rb)
    np.testing.assert_array_equal(oa["thetas"][3], ob["thetas"][3])
    np.testing.assert_allclose(ob["thetas"][4] - ob["thetas"][3], 0.5 * (oa["thetas"][4] - oa["thetas"][3]), rtol=1e-12)
