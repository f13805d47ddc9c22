"""Pins of the oracle's dense layer and softmax cross-entropy (the units of the paper's classifier
MLP_CLS, classifier equation, and of its loss equation) against things other than the oracle:
closed forms, invariants, a library cross-check (torch CPU fp64 autograd) and finite differences."""
import math

import numpy as np
import pytest
import torch

import oracle

RNG = np.random.default_rng(20240811)


def test_ce_uniform_logits_is_log_c():
    # all logits equal -> softmax is uniform -> loss = ln C whatever the labels are
    for c in (2, 8, 41, 64):
        n = 37
        loss, g = oracle.softmax_ce(np.full((n, c), 3.25), RNG.integers(0, c, n))
        assert abs(loss - math.log(c)) < 1e-14
        assert np.allclose(g.sum(axis=1), 0.0, atol=1e-16)


def test_ce_two_class_closed_form():
    # two classes, logits (a, b), label 0: loss = log(1 + exp(b - a)); gradient wrt a = -sigmoid(b - a) / n
    a, b = 0.7, -1.9
    loss, g = oracle.softmax_ce(np.array([[a, b]]), np.array([0]))
    assert abs(loss - math.log1p(math.exp(b - a))) < 1e-15
    s = 1.0 / (1.0 + math.exp(-(b - a)))
    assert np.allclose(g, [[-s, s]], atol=1e-15)


def test_ce_shift_invariance_and_large_logits():
    n, c = 50, 13
    x = RNG.normal(size=(n, c)) * 5
    y = RNG.integers(0, c, n)
    l0, g0 = oracle.softmax_ce(x, y)
    l1, g1 = oracle.softmax_ce(x + RNG.normal(size=(n, 1)) * 100, y)  # a per-row shift changes nothing
    assert abs(l0 - l1) < 1e-12 and np.allclose(g0, g1, atol=1e-13)
    big, _ = oracle.softmax_ce(np.array([[1000.0, 0.0], [0.0, 1000.0]]), np.array([0, 0]))
    assert abs(big - 500.0) < 1e-9  # (0 + 1000) / 2, no overflow


def test_ce_matches_torch_fp64():
    n, c = 301, 47
    x = RNG.normal(size=(n, c)) * 2
    y = RNG.integers(0, c, n)
    loss, g = oracle.softmax_ce(x, y)
    xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    lt = torch.nn.functional.cross_entropy(xt, torch.tensor(y, dtype=torch.int64), reduction="mean")
    lt.backward()
    assert abs(loss - lt.item()) < 1e-13
    assert np.allclose(g, xt.grad.numpy(), atol=1e-15, rtol=1e-12)


def test_ce_rejects_bad_label():
    with pytest.raises(ValueError):
        oracle.softmax_ce(np.zeros((3, 4)), np.array([0, 4, 1]))


@pytest.mark.parametrize("act", [0, 1])
@pytest.mark.parametrize("bias", [False, True])
def test_linear_matches_torch_fp64_autograd(act, bias):
    n, w_in, w_out = 67, 19, 23
    X = RNG.normal(size=(n, w_in)); W = RNG.normal(size=(w_in, w_out)) / 4
    b = RNG.normal(size=w_out) / 3 if bias else None
    dY = RNG.normal(size=(n, w_out))
    Y, P = oracle.linear_fwd(X, W, b, act)
    Xt = torch.tensor(X, requires_grad=True); Wt = torch.tensor(W, requires_grad=True)
    bt = torch.tensor(b, requires_grad=True) if bias else None
    Pt = Xt @ Wt + (bt if bias else 0.0)
    Yt = torch.relu(Pt) if act else Pt
    assert np.allclose(Y, Yt.detach().numpy(), atol=1e-13)
    Yt.backward(torch.tensor(dY))
    mask = (P > 0) if act else np.ones_like(P, dtype=bool)
    g = oracle.linear_bwd(X, W, mask, dY)
    assert np.allclose(g["dX"], Xt.grad.numpy(), atol=1e-12)
    assert np.allclose(g["dW"], Wt.grad.numpy(), atol=1e-12)
    if bias:
        assert np.allclose(g["db"], bt.grad.numpy(), atol=1e-12)


def test_linear_hand_example():
    # one row, two inputs, two outputs, ReLU: P = [1*2 + 3*(-1) + 0.5, 1*0 + 3*1 - 1] = [-0.5, 2]
    X = np.array([[1.0, 3.0]]); W = np.array([[2.0, 0.0], [-1.0, 1.0]]); b = np.array([0.5, -1.0])
    Y, P = oracle.linear_fwd(X, W, b, act=1)
    assert np.array_equal(P, [[-0.5, 2.0]]) and np.array_equal(Y, [[0.0, 2.0]])
    g = oracle.linear_bwd(X, W, P > 0, np.array([[10.0, 100.0]]))
    assert np.array_equal(g["db"], [0.0, 100.0])
    assert np.array_equal(g["dW"], [[0.0, 100.0], [0.0, 300.0]])
    assert np.array_equal(g["dX"], [[0.0, 100.0]])


def test_classifier_chain_finite_differences():
    """loss(H) = CE(relu(H W1 + b1) W2 + b2): the oracle's analytic dH against central differences of
    its own fp64 forward, away from ReLU kinks."""
    n, d, h, c = 9, 6, 7, 5
    H = RNG.normal(size=(n, d)); W1 = RNG.normal(size=(d, h)) / 2; b1 = RNG.normal(size=h) / 2
    W2 = RNG.normal(size=(h, c)) / 2; b2 = RNG.normal(size=c) / 2
    y = RNG.integers(0, c, n)

    def fwd(Hx):
        A, P = oracle.linear_fwd(Hx, W1, b1, act=1)
        logits, _ = oracle.linear_fwd(A, W2, b2, act=0)
        return oracle.softmax_ce(logits, y, want_grad=False)[0], A, P, logits

    loss, A, P, logits = fwd(H)
    assert np.abs(P).min() > 1e-4  # no pre-activation near the kink
    _, dlog = oracle.softmax_ce(logits, y)
    g2 = oracle.linear_bwd(A, W2, np.ones_like(logits, dtype=bool), dlog)
    g1 = oracle.linear_bwd(H, W1, P > 0, g2["dX"])
    eps = 1e-6
    num = np.zeros_like(H)
    for i in range(n):
        for j in range(d):
            Hp = H.copy(); Hp[i, j] += eps
            Hm = H.copy(); Hm[i, j] -= eps
            num[i, j] = (fwd(Hp)[0] - fwd(Hm)[0]) / (2 * eps)
    assert np.allclose(g1["dX"], num, atol=1e-9)


def test_linear_adjoint_identity():
    # <X W, G> = <X, G W^T> pins the transposed product of the backward pass
    n, w_in, w_out = 31, 11, 17
    X = RNG.normal(size=(n, w_in)); W = RNG.normal(size=(w_in, w_out)); G = RNG.normal(size=(n, w_out))
    Y, _ = oracle.linear_fwd(X, W)
    g = oracle.linear_bwd(X, W, np.ones((n, w_out), dtype=bool), G)
    assert abs((Y * G).sum() - (X * g["dX"]).sum()) < 1e-10 * np.abs(Y * G).sum()
