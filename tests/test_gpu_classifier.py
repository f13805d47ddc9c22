"""GPU parity of the dense layer and the softmax cross-entropy (the units of the paper's classifier
MLP_CLS and loss equation) against the fp64 CPU oracle on the same seeded inputs: fp32 outputs and
gradients within a max relative error of 1e-4 (max|got - want| / max|want|)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2408_11500_amd import binding as B
from gpu_util import TOL, assert_close, dev, pack_mask, padded, unpack_mask

pytestmark = pytest.mark.gpu


def ws_tensor(nbytes):
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")


SHAPES = [(1, 1, 1), (5, 3, 2), (130, 32, 32), (1000, 25, 64), (2049, 64, 47), (700, 256, 256), (333, 100, 130),
          (4100, 256, 40), (257, 301, 33)]


@pytest.mark.parametrize("n,w_in,w_out", SHAPES)
@pytest.mark.parametrize("act", [B.ACT_NONE, B.ACT_RELU])
@pytest.mark.parametrize("bias", [True, False])
def test_linear_fwd_bwd_parity(n, w_in, w_out, act, bias):
    rng = np.random.default_rng(n * 131 + w_in * 7 + w_out + act)
    X = rng.normal(size=(n, w_in)).astype(np.float32)
    W = (rng.normal(size=(w_in, w_out)) / np.sqrt(w_in)).astype(np.float32)
    b = (rng.normal(size=w_out) / 4).astype(np.float32) if bias else None
    dY = rng.normal(size=(n, w_out)).astype(np.float32)
    Yo, Po = oracle.linear_fwd(X, W, b, act)

    ldx = (w_in + 3) // 4 * 4 + 4
    Xd = padded(X, ldx)
    Yfull = torch.full((n, w_out + 3), 7.0, dtype=torch.float32, device="cuda")  # odd ld, sentinel padding
    Yd = Yfull[:, :w_out]
    mw = (w_out + 31) // 32
    mask = torch.zeros((n, mw), dtype=torch.int32, device="cuda") if act else None
    B.slicegcn_linear_fwd(Xd, dev(W), dev(b) if bias else None, Yd, mask, act=act)
    torch.cuda.synchronize()
    assert_close(Yd.cpu().numpy(), Yo, "Y")
    assert torch.all(Yfull[:, w_out:] == 7.0)  # padding untouched
    if act:
        got = unpack_mask(mask.cpu().numpy(), w_out)
        band = 1e-5 * np.sqrt(np.mean(Po ** 2))
        differ = got != (Po > 0)
        assert not np.any(differ & (np.abs(Po) > band)), "activation pattern differs outside the rounding band"
        mask_o = (Po > 0)
        mask_d = dev(pack_mask(mask_o.astype(np.uint8)), torch.int32)  # both sides differentiate the oracle's pattern
    else:
        mask_o = np.ones((n, w_out), dtype=bool)
        mask_d = None
    go = oracle.linear_bwd(X, W, mask_o, dY)
    dX = torch.empty((n, w_in + 1), dtype=torch.float32, device="cuda")[:, :w_in]
    dW = torch.empty((w_in, w_out), dtype=torch.float32, device="cuda")
    db = torch.empty(w_out, dtype=torch.float32, device="cuda")
    ws = ws_tensor(B.slicegcn_linear_bwd_workspace_bytes(n, w_in, w_out))
    B.slicegcn_linear_bwd(Xd, dev(W), mask_d, padded(dY, w_out + 5), dX, dW, db, ws, act=act)
    torch.cuda.synchronize()
    assert_close(dX.cpu().numpy(), go["dX"], "dX")
    assert_close(dW.cpu().numpy(), go["dW"], "dW")
    assert_close(db.cpu().numpy(), go["db"], "db")
    # skipping outputs: only dX, no workspace
    dX2 = torch.empty((n, w_in), dtype=torch.float32, device="cuda")
    B.slicegcn_linear_bwd(Xd, dev(W), mask_d, dev(dY), dX2, None, None, None, act=act)
    torch.cuda.synchronize()
    assert_close(dX2.cpu().numpy(), go["dX"], "dX alone")


@pytest.mark.parametrize("n,c", [(1, 1), (1, 2), (3, 8), (64, 40), (65, 41), (1000, 47), (4097, 64), (300, 100), (77, 17)])
def test_softmax_ce_parity(n, c):
    rng = np.random.default_rng(n * 17 + c)
    x = (rng.normal(size=(n, c)) * 3).astype(np.float32)
    y = rng.integers(0, c, n)
    lo, go = oracle.softmax_ce(x, y)
    xd = padded(x, c + 3)
    g = torch.full((n, c + 2), 9.0, dtype=torch.float32, device="cuda")
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    ws = ws_tensor(B.slicegcn_softmax_ce_workspace_bytes(n))
    B.slicegcn_softmax_ce(xd, dev(y, torch.int32), loss, g[:, :c], ws)
    torch.cuda.synchronize()
    assert abs(loss.item() - lo) <= TOL * abs(lo) + 1e-7
    assert_close(g[:, :c].cpu().numpy(), go, "dlogits")
    assert torch.all(g[:, c:] == 9.0)
    # loss only, and bitwise reproducible
    loss2 = torch.zeros(1, dtype=torch.float32, device="cuda")
    B.slicegcn_softmax_ce(xd, dev(y, torch.int32), loss2, None, ws)
    assert loss2.item() == loss.item()


def test_softmax_ce_extreme_logits_and_bad_label():
    x = np.array([[1000.0, 0.0], [0.0, 1000.0], [-1000.0, -1000.0]], dtype=np.float32)
    y = np.array([0, 0, 1])
    lo, go = oracle.softmax_ce(x, y)
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    g = torch.empty((3, 2), dtype=torch.float32, device="cuda")
    ws = ws_tensor(B.slicegcn_softmax_ce_workspace_bytes(3))
    B.slicegcn_softmax_ce(dev(x), dev(y, torch.int32), loss, g, ws)
    assert abs(loss.item() - lo) <= 1e-4 * lo and np.allclose(g.cpu().numpy(), go, atol=1e-7)
    B.slicegcn_softmax_ce(dev(x), dev(np.array([0, 2, 1]), torch.int32), loss, g, ws)  # label 2 of 2 classes
    assert np.isnan(loss.item())


def test_linear_rejects_bad_arguments():
    X = torch.zeros((4, 8), dtype=torch.float32, device="cuda")
    W = torch.zeros((8, 8), dtype=torch.float32, device="cuda")
    Y = torch.zeros((4, 8), dtype=torch.float32, device="cuda")
    with pytest.raises(B.SliceGCNError) as e:
        B.slicegcn_linear_fwd(X, W, None, Y, None, act=B.ACT_RELU)  # ReLU without a mask
    assert e.value.status == B.EINVAL
    with pytest.raises(B.SliceGCNError) as e:
        B.slicegcn_linear_bwd(X, W, None, Y, None, W.clone(), None, None)  # dW wanted, no workspace
    assert e.value.status == B.EWORKSPACE


def test_classifier_chain_at_workload_shape():
    """MLP_CLS + loss at the citation-graph shape (N = 169 343, 4 slices x 64 -> 256 -> 40 classes):
    forward and backward through the C ABI against the oracle."""
    import synth
    from synth import configs
    w = synth.WORKLOADS["cfg2"]
    n, h, c = w.n_nodes, w.hidden, w.classes
    H = configs.normal_matrix(w.seed, 11, n, h).numpy()
    rng = np.random.default_rng(3)
    W1 = (rng.uniform(-1, 1, size=(h, h)) * np.sqrt(6 / (2 * h))).astype(np.float32)
    b1 = (rng.normal(size=h) * 0.1).astype(np.float32)
    W2 = (rng.uniform(-1, 1, size=(h, c)) * np.sqrt(6 / (h + c))).astype(np.float32)
    b2 = (rng.normal(size=c) * 0.1).astype(np.float32)
    y = configs.labels(w).numpy()
    Ao, P1 = oracle.linear_fwd(H, W1, b1, act=1)
    Lo, _ = oracle.linear_fwd(Ao, W2, b2, act=0)
    lo, dLo = oracle.softmax_ce(Lo, y)

    f32 = dict(dtype=torch.float32, device="cuda")
    Hd = dev(H)
    A = torch.empty((n, h), **f32); logits = torch.empty((n, c), **f32)
    mask = torch.zeros((n, (h + 31) // 32), dtype=torch.int32, device="cuda")
    B.slicegcn_linear_fwd(Hd, dev(W1), dev(b1), A, mask, act=B.ACT_RELU)
    B.slicegcn_linear_fwd(A, dev(W2), dev(b2), logits, None, act=B.ACT_NONE)
    loss = torch.zeros(1, **f32); dlog = torch.empty((n, c), **f32)
    ws = ws_tensor(max(B.slicegcn_softmax_ce_workspace_bytes(n), B.slicegcn_linear_bwd_workspace_bytes(n, h, h)))
    B.slicegcn_softmax_ce(logits, dev(y, torch.int32), loss, dlog, ws)
    assert_close(A.cpu().numpy(), Ao, "A1")
    assert_close(logits.cpu().numpy(), Lo, "logits")
    assert abs(loss.item() - lo) <= TOL * lo
    assert_close(dlog.cpu().numpy(), dLo, "dlogits")
    # backward with the oracle's activation pattern on both sides
    g2 = oracle.linear_bwd(Ao, W2, np.ones((n, c), dtype=bool), dLo)
    g1 = oracle.linear_bwd(H, W1, P1 > 0, g2["dX"])
    mask_o = dev(pack_mask((P1 > 0).astype(np.uint8)), torch.int32)
    dA = torch.empty((n, h), **f32); dH = torch.empty((n, h), **f32)
    dW2 = torch.empty((h, c), **f32); db2 = torch.empty(c, **f32); dW1 = torch.empty((h, h), **f32); db1 = torch.empty(h, **f32)
    B.slicegcn_linear_bwd(dev(Ao), dev(W2), None, dev(dLo), dA, dW2, db2, ws, act=B.ACT_NONE)
    B.slicegcn_linear_bwd(Hd, dev(W1), mask_o, dA, dH, dW1, db1, ws, act=B.ACT_RELU)
    torch.cuda.synchronize()
    for got, want, what in ((dA, g2["dX"], "dA1"), (dW2, g2["dW"], "dW2"), (db2, g2["db"], "db2"),
                            (dH, g1["dX"], "dH"), (dW1, g1["dW"], "dW1"), (db1, g1["db"], "db1")):
        assert_close(got.cpu().numpy(), want, what)
