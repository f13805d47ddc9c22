"""Parameter shapes of a SliceGCN model and seeded weights for them (inputs only).

Per slice and per layer there is an aggregation weight with its bias (inside the activation)
and a self weight with its bias (outside it); the slice encoding is one row per slice; the
classifier is Linear(k*h -> hidden) followed by Linear(hidden -> classes).  This reading of
the paper's layer equation is the one that reproduces its printed parameter-count table.
"""
from __future__ import annotations

import torch

from . import configs, rng


def layer_widths(first_in: int, slice_hidden: int, layers: int):
    """[(w_in, w_out)] of the layers of one slice's GCN."""
    return [(first_in if l == 0 else slice_hidden, slice_hidden) for l in range(layers)]


def param_shapes(feat: int, classes: int, layers: int, p: int, hidden: int, first_in: int,
                 slice_hidden: int, slice_encoding: bool = False, feature_fusion: bool = False):
    """Every parameter tensor of the model as a list of (name, shape)."""
    shapes = []
    for i in range(p):
        for l, (wi, wo) in enumerate(layer_widths(first_in, slice_hidden, layers)):
            shapes += [(f"s{i}.l{l}.W_agg", (wi, wo)), (f"s{i}.l{l}.b", (wo,)),
                       (f"s{i}.l{l}.W_self", (wi, wo)), (f"s{i}.l{l}.b_self", (wo,))]
    if slice_encoding:
        shapes.append(("E", (p, slice_hidden)))
    if feature_fusion:
        shapes += [("ff.W0", (feat, feat)), ("ff.b0", (feat,)), ("ff.W1", (feat, first_in)), ("ff.b1", (first_in,))]
    shapes += [("cls.W0", (p * slice_hidden, hidden)), ("cls.b0", (hidden,)),
               ("cls.W1", (hidden, classes)), ("cls.b1", (classes,))]
    return shapes


def param_count(shapes) -> int:
    total = 0
    for _, shp in shapes:
        c = 1
        for d in shp:
            c *= d
        total += c
    return total


def slice_layer_params(w: configs.Workload, slice_id: int, layer: int, w_in: int, w_out: int, device="cpu",
                       bias_std: float = 0.0):
    """Seeded Glorot weights; biases are zero unless ``bias_std`` asks for visible ones (tests)."""
    tag = (slice_id * 64 + layer) * 4
    W_agg = configs.glorot(w.seed, tag, w_in, w_out, device)
    W_self = configs.glorot(w.seed, tag + 1, w_in, w_out, device)
    if bias_std > 0:
        j = rng.arange64(w_out, device)
        b = (rng.normal(w.seed, configs.STREAM_W, j + ((tag + 2) << 32)) * bias_std).to(torch.float32)
        b_self = (rng.normal(w.seed, configs.STREAM_W, j + ((tag + 3) << 32)) * bias_std).to(torch.float32)
    else:
        b = torch.zeros(w_out, dtype=torch.float32, device=device)
        b_self = torch.zeros(w_out, dtype=torch.float32, device=device)
    return W_agg, b, W_self, b_self


def classifier_params(w: configs.Workload, width: int, device="cpu", bias_std: float = 0.0):
    """Seeded Glorot weights of the classifier MLP (width -> hidden -> classes); biases as above."""
    tag = 1 << 20
    W1 = configs.glorot(w.seed, tag, width, w.hidden, device)
    W2 = configs.glorot(w.seed, tag + 1, w.hidden, w.classes, device)
    if bias_std > 0:
        b1 = (rng.normal(w.seed, configs.STREAM_W, rng.arange64(w.hidden, device) + ((tag + 2) << 32)) * bias_std).to(torch.float32)
        b2 = (rng.normal(w.seed, configs.STREAM_W, rng.arange64(w.classes, device) + ((tag + 3) << 32)) * bias_std).to(torch.float32)
    else:
        b1 = torch.zeros(w.hidden, dtype=torch.float32, device=device)
        b2 = torch.zeros(w.classes, dtype=torch.float32, device=device)
    return W1, b1, W2, b2


def fusion_params(w: configs.Workload, out_width: int, device="cpu", bias_std: float = 0.0):
    """Seeded Glorot weights of the feature-fusion MLP (feat -> feat -> out_width); biases as above."""
    tag = (1 << 20) + 16
    W1 = configs.glorot(w.seed, tag, w.feat, w.feat, device)
    W2 = configs.glorot(w.seed, tag + 1, w.feat, out_width, device)
    if bias_std > 0:
        b1 = (rng.normal(w.seed, configs.STREAM_W, rng.arange64(w.feat, device) + ((tag + 2) << 32)) * bias_std).to(torch.float32)
        b2 = (rng.normal(w.seed, configs.STREAM_W, rng.arange64(out_width, device) + ((tag + 3) << 32)) * bias_std).to(torch.float32)
    else:
        b1 = torch.zeros(w.feat, dtype=torch.float32, device=device)
        b2 = torch.zeros(out_width, dtype=torch.float32, device=device)
    return W1, b1, W2, b2
