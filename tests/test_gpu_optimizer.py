"""GPU parity of the Adam step against the fp64 oracle, and a short training run of the whole model
(slice stack + classifier + loss + optimiser) that has to reduce the loss."""
import numpy as np
import pytest
import torch

import oracle
import synth
from synth import configs, model
import paper_2408_11500_amd as sg
from paper_2408_11500_amd import binding as B
from paper_2408_11500_amd.stack import Classifier, Optimizer, SliceStack
from gpu_util import assert_close, dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("count", [1, 255, 4097, 100003])
@pytest.mark.parametrize("wd", [0.0, 0.01])
def test_adam_step_parity(count, wd):
    rng = np.random.default_rng(count)
    p = rng.normal(size=count); m = np.zeros(count); v = np.zeros(count)
    pd, md, vd = dev(p), dev(m), dev(v)
    for t in range(1, 6):
        g = (rng.normal(size=count) * t).astype(np.float32)
        lr = oracle.cosine_lr(1e-2, 1e-4, t - 1, 5)
        oracle.adam_step(p, g.astype(np.float64), m, v, lr, t, weight_decay=wd)
        B.slicegcn_adam_step(pd, dev(g), md, vd, lr, t, weight_decay=wd)
        assert_close(pd.cpu().numpy(), p, f"param after step {t}", tol=1e-5)
        assert_close(md.cpu().numpy(), m, "m", tol=1e-5)
        assert_close(vd.cpu().numpy(), v, "v", tol=1e-5)


def test_adam_rejects_bad_arguments():
    t = torch.zeros(8, dtype=torch.float32, device="cuda")
    with pytest.raises(B.SliceGCNError):
        B.slicegcn_adam_step(t, t.clone(), t.clone(), t.clone(), 1e-3, 0)          # step < 1
    with pytest.raises(B.SliceGCNError):
        B.slicegcn_adam_step(t, t.clone(), t.clone(), t.clone(), 1e-3, 1, beta1=1.0)


def make_trainer(w, g, X, y, use_ff, graph_replay=False):
    from paper_2408_11500_amd.train import SliceGCNTrainer
    tr = SliceGCNTrainer(g, X, y, w.k, w.slice_hidden, w.layers, w.hidden, w.classes, use_ff=use_ff,
                         graph_replay=graph_replay)
    for i in range(w.k):
        for l, (wi, wo) in enumerate(tr.stack.widths):
            tr.stack.set_params(i, l, *model.slice_layer_params(w, i, l, wi, wo))
    tr.cls.set_params(*model.classifier_params(w, w.k * w.slice_hidden))
    if use_ff:
        tr.ff.set_params(*model.fusion_params(w, tr.ff.s))
    tr.start(1e-2, 1e-4, 60)
    return tr


@pytest.mark.parametrize("use_ff", [False, True])
def test_training_with_graph_replay_equals_eager(use_ff):
    """Replaying forward + loss + backward as one HIP graph gives, epoch after epoch, the same bits as the
    eager call sequence (the parameter update runs eagerly between the replays in both)."""
    w = synth.WORKLOADS["cfg1"]
    s_, d_ = configs.edges(w)
    g = sg.slicegcn_build_norm_csr(s_.cuda(), d_.cuda(), w.n_nodes)
    X = configs.features(w).cuda()
    y = X[:, :w.classes].argmax(dim=1)
    eager = make_trainer(w, g, X, y, use_ff)
    replay = make_trainer(w, g, X, y, use_ff, graph_replay=True)
    for t in range(6):
        le, lr_ = eager.epoch(t), replay.epoch(t)
        torch.cuda.synchronize()
        assert torch.equal(le, lr_), t
        assert torch.equal(eager.opt.P, replay.opt.P), t
    g.destroy()


@pytest.mark.parametrize("use_ff", [False, True])
def test_training_reduces_the_loss(use_ff):
    """The training algorithm end to end on the tiny workload (direct slicing and feature fusion) with
    labels that depend on the features: forward, loss, backward and an Adam step per epoch; the loss must
    at least halve."""
    from paper_2408_11500_amd.train import SliceGCNTrainer
    w = synth.WORKLOADS["cfg1"]
    s_, d_ = configs.edges(w)
    g = sg.slicegcn_build_norm_csr(s_.cuda(), d_.cuda(), w.n_nodes)
    X = configs.features(w).cuda()
    y = X[:, :w.classes].argmax(dim=1)   # learnable: the largest of the first C features
    tr = SliceGCNTrainer(g, X, y, w.k, w.slice_hidden, w.layers, w.hidden, w.classes, use_ff=use_ff)
    for i in range(w.k):
        for l, (wi, wo) in enumerate(tr.stack.widths):
            tr.stack.set_params(i, l, *model.slice_layer_params(w, i, l, wi, wo))
    tr.cls.set_params(*model.classifier_params(w, w.k * w.slice_hidden))
    if use_ff:
        tr.ff.set_params(*model.fusion_params(w, tr.ff.s))
    tr.start(1e-2, 1e-4, 60)
    assert tr.stack.params[0][0]["W_agg"].data_ptr() >= tr.opt.P.data_ptr()   # rebound to views of the flat buffer
    losses = [tr.epoch(t).item() for t in range(60)]
    assert np.isfinite(losses).all()
    assert losses[-1] < 0.5 * losses[0], losses[::10]
    g.destroy()
