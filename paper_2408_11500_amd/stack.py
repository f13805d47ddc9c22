"""Call sequence of one full-batch pass over k feature slices (the inner loops of the paper's
training algorithm): for every slice, L layer evaluations, then slice encoding + CONCAT, and
the same chain backwards.  This module only owns buffers (torch device tensors) and orders the
library calls; every arithmetic step is a kernel of ``libslicegcn.so``.
"""
from __future__ import annotations

import torch

from . import binding as B


def padded_ld(width: int) -> int:
    """Leading dimension for a slice operand: every row starts on a 128-byte boundary, so a gathered
    row (or a column pass over it) touches the fewest cache lines (a 301-wide slice at ld 304 has
    every other row straddle one line more: 8.7 vs 7.8 ms per aggregation)."""
    return (width + 31) // 32 * 32


class SliceStack:
    def __init__(self, graph: B.Graph, n_nodes: int, k: int, first_width: int, slice_hidden: int, layers: int,
                 device="cuda", slice_encoding: bool = True, act_last: int = B.ACT_RELU,
                 shared_input: torch.Tensor | None = None, cache_first_aggregation: bool = False,
                 fuse_encoding: bool = True, order: int = 0, scaled: bool | None = None, streams: int = 1):
        """``shared_input``: with feature fusion every slice model reads the same fused n x first_width
        matrix; the stack then also returns the gradient with respect to it (``dXin``).
        ``order``: 0 (aggregate first), LAYER_TRANSFORM_FIRST or LAYER_ORDER_AUTO, applied to every layer.
        ``scaled``: keep the activations between aggregate-first layers as D~^-1/2 H (the layer flags IN_SCALED /
        OUT_SCALED), so that no aggregation reads the stored values; the raw slices are then scaled once by
        ``prepare_inputs`` (call it after filling ``X``).  None = by graph size: the layout pays where the
        aggregation streams the stored entries from memory (measured: -3 % per step at 126 M and 310 M entries) and
        costs a little where the whole graph sits in cache and the dense kernels' extra row factors show
        (+3 % at 2.5 M entries), so it is used from 16 M stored entries on.
        ``streams``: how many slice models run at a time, each on a HIP stream of its own (the slice models are
        independent between the raw features and the concatenation, and a graph handle is read-only, so they only
        need workspaces of their own).  1 = one after the other on the caller's stream.  More pays on small graphs,
        whose kernels leave most of the chip idle; every slice computes exactly what it computes alone, so results
        are bitwise the same."""
        self.g, self.n, self.k, self.L = graph, n_nodes, k, layers
        self.w0, self.hs = first_width, slice_hidden
        self.dev = torch.device(device)
        self.act_last = act_last
        f32 = dict(dtype=torch.float32, device=self.dev)
        self.widths = [(first_width if l == 0 else slice_hidden, slice_hidden) for l in range(layers)]
        self.order = order
        if scaled is None:
            scaled = graph.view().nnz >= (1 << 24)
        self.scaled = scaled
        # layers that run in the transform-first order keep no aggregation of their input
        self.tf = [order == B.LAYER_TRANSFORM_FIRST or (order == B.LAYER_ORDER_AUTO and wo < wi) for wi, wo in self.widths]
        # layout flags per layer: a layer reads a scaled input when its producer could write one (the previous layer if
        # both run aggregate-first; the raw slice, scaled in place by prepare_inputs, for the first layer)
        shared = shared_input is not None
        self.in_scaled = [scaled and not self.tf[l] and (not shared if l == 0 else not self.tf[l - 1]) for l in range(layers)]
        self.layout = [(B.LAYER_IN_SCALED if self.in_scaled[l] else 0) |
                       (B.LAYER_OUT_SCALED if l + 1 < layers and self.in_scaled[l + 1] else 0) for l in range(layers)]
        self.inputs_prepared = False
        # inputs
        # with direct slicing the first layer aggregates constant features: A^ X_s can be kept across passes
        # (the paper's implementation recomputes it; off by default so that a pass measures every kernel)
        self.cache_first = cache_first_aggregation and shared_input is None and not self.tf[0]
        self.first_valid = [False] * k
        self.shared = shared_input is not None
        self.X = ([shared_input] * k if self.shared
                  else [torch.zeros((n_nodes, padded_ld(first_width)), **f32) for _ in range(k)])
        self.dXin = torch.empty((n_nodes, padded_ld(first_width)), **f32) if self.shared else None
        self.dXtmp = torch.empty((n_nodes, padded_ld(first_width)), **f32) if self.shared and k > 1 else None
        # parameters and their gradients: [slice][layer] -> dict
        self.params = [[None] * layers for _ in range(k)]
        self.grads = [[None] * layers for _ in range(k)]
        self.E = torch.zeros((k, slice_hidden), **f32) if slice_encoding else None
        self.dE = torch.zeros((k, slice_hidden), **f32) if slice_encoding else None
        # activations kept for the backward pass
        self.H = [[torch.empty((n_nodes, padded_ld(slice_hidden)), **f32) for _ in range(layers - 1)] for _ in range(k)]
        self.Z = [[None if self.tf[l] else torch.empty((n_nodes, padded_ld(wi)), **f32) for l, (wi, _) in enumerate(self.widths)]
                  for _ in range(k)]
        mw = (slice_hidden + 31) // 32
        self.mask = [[torch.zeros((n_nodes, mw), dtype=torch.int32, device=self.dev) for _ in range(layers)] for _ in range(k)]
        self.Hcat = torch.empty((n_nodes, k * slice_hidden), **f32)
        # Slice encoding adds the row vector E[i] to every node row of slice i; the last layer's self-term bias does
        # the same, so E[i] can ride on it: the last layer then stores the encoded output straight into its column
        # block (no encoding pass) and dE[i] is that layer's db_self (no column-sum pass over dH).
        self.fuse_encoding = fuse_encoding and slice_encoding
        self.b_eff = torch.zeros((k, slice_hidden), **f32) if self.fuse_encoding else None
        # slice i runs on lane i mod lanes; a lane has its own stream, workspace and backward scratch
        self.lanes = max(1, min(k, int(streams)))
        self.streams = [torch.cuda.Stream(device=self.dev) for _ in range(self.lanes)] if self.lanes > 1 else []
        self.dbuf = [[torch.empty((n_nodes, padded_ld(slice_hidden)), **f32) for _ in range(2)] if layers > 1 else []
                     for _ in range(self.lanes)]
        # with a shared (learned) input and several lanes every slice keeps its own input gradient until the lanes
        # have joined; they are then added in slice order, as the one-lane pass adds them
        self.dXs = ([torch.empty((n_nodes, padded_ld(first_width)), **f32) for _ in range(k - 1)]
                    if self.shared and self.lanes > 1 else [])
        ws = 0
        for l, (wi, wo) in enumerate(self.widths):
            ws = max(ws, B.slicegcn_layer_fwd_workspace_bytes(graph, wi, wo, order),
                     B.slicegcn_layer_bwd_workspace_bytes(graph, wi, wo, l > 0 or self.shared, order))
        ws = max(ws, B.slicegcn_concat_bwd_workspace_bytes(n_nodes, [slice_hidden] * k))
        self.ws_lane = [torch.empty(ws, dtype=torch.uint8, device=self.dev) for _ in range(self.lanes)]
        self.ws = self.ws_lane[0]

    # ---------------------------------------------------------------------------------
    def set_params(self, i: int, l: int, W_agg, b, W_self, b_self):
        wi, wo = self.widths[l]
        f32 = dict(dtype=torch.float32, device=self.dev)
        self.params[i][l] = dict(W_agg=W_agg.to(**f32).contiguous(), b=b.to(**f32).contiguous(),
                                 W_self=None if W_self is None else W_self.to(**f32).contiguous(),
                                 b_self=None if b_self is None else b_self.to(**f32).contiguous())
        self.grads[i][l] = dict(dW_agg=torch.empty((wi, wo), **f32), db=torch.empty(wo, **f32),
                                dW_self=torch.empty((wi, wo), **f32) if W_self is not None else None,
                                db_self=torch.empty(wo, **f32) if W_self is not None else None)

    def parameter_slots(self):
        """(holder of the parameter, key, holder of its gradient, key) for every learnable tensor."""
        out = []
        for i in range(self.k):
            for l in range(self.L):
                for pn, gn in (("W_agg", "dW_agg"), ("b", "db"), ("W_self", "dW_self"), ("b_self", "db_self")):
                    if self.params[i][l][pn] is not None:
                        out.append((self.params[i][l], pn, self.grads[i][l], gn))
        if self.E is not None:
            out.append((self, "E", self, "dE"))
        return out

    def inputs_changed(self):
        """Call after writing new features into ``X``: cached first-layer aggregations are dropped."""
        self.first_valid = [False] * self.k
        self.inputs_prepared = False

    def prepare_inputs(self):
        """Once per set of raw features: with the scaled layout the slices in ``X`` become D~^-1/2 X_s, in place."""
        if self.in_scaled[0] and not self.shared and not self.inputs_prepared:
            for x in self.X:
                B.slicegcn_scale_rows(self.g, x[:, :self.w0], x, width=self.w0)
        self.inputs_prepared = True

    def hin(self, i: int, l: int) -> torch.Tensor:
        wi = self.widths[l][0]
        return (self.X[i] if l == 0 else self.H[i][l - 1])[:, :wi]

    def hout(self, i: int, l: int) -> torch.Tensor:
        if l == self.L - 1:
            return self.Hcat[:, i * self.hs:(i + 1) * self.hs]
        return self.H[i][l][:, :self.hs]

    def zbuf(self, i: int, l: int):
        return None if self.tf[l] else self.Z[i][l][:, :self.widths[l][0]]

    def act(self, l: int) -> int:
        return self.act_last if l == self.L - 1 else B.ACT_RELU

    # ---------------------------------------------------------------------------------
    def encoding_fused(self) -> bool:
        last = self.L - 1
        return self.fuse_encoding and all(self.params[i][last]["W_self"] is not None and
                                          self.params[i][last]["b_self"] is not None for i in range(self.k))

    def forward_slice(self, i: int):
        if not self.inputs_prepared:
            self.prepare_inputs()
        fused = self.encoding_fused()
        for l in range(self.L):
            p = self.params[i][l]
            wi = self.widths[l][0]
            b_self = p["b_self"]
            if fused and l == self.L - 1:  # b_self + E[i], two tiny launches
                b_self = self.b_eff[i]
                B.slicegcn_slice_feature(p["b_self"].view(1, -1), 0, self.hs, b_self.view(1, -1))
                B.slicegcn_accumulate(b_self.view(1, -1), self.E[i].view(1, -1))
            B.slicegcn_layer_fwd(self.g, self.hin(i, l), p["W_agg"], p["b"], p["W_self"], b_self, self.hout(i, l),
                                 self.zbuf(i, l), self.mask[i][l], act=self.act(l),
                                 z_valid=l == 0 and self.cache_first and self.first_valid[i], ws=self.ws_lane[i % self.lanes],
                                 order=self.order, layout=self.layout[l])
        self.first_valid[i] = True

    def _on_lanes(self, fn):
        """fn(i) for every slice: in turn on the caller's stream, or slice i on lane i mod lanes, the lanes
        starting after what the caller's stream holds so far and the caller's stream going on after all of them."""
        if self.lanes == 1:
            for i in range(self.k):
                fn(i)
            return
        main = torch.cuda.current_stream()
        for s in self.streams:
            s.wait_stream(main)
        for i in range(self.k):
            with torch.cuda.stream(self.streams[i % self.lanes]):
                fn(i)
        for s in self.streams:
            main.wait_stream(s)

    def forward(self) -> torch.Tensor:
        if not self.inputs_prepared:
            self.prepare_inputs()
        self._on_lanes(self.forward_slice)
        # the last layer of every slice already stored into its column block: encode in place, unless that is done
        if not self.encoding_fused():
            B.slicegcn_concat([self.hout(i, self.L - 1) for i in range(self.k)], self.E, self.Hcat)
        return self.Hcat

    def backward(self, dH: torch.Tensor):
        fused = self.encoding_fused()
        if self.E is not None and not fused:
            B.slicegcn_concat_bwd(dH, [self.hs] * self.k, dE=self.dE, ws=self.ws)
        deferred = self.shared and self.lanes > 1   # the slices' input gradients are added after the lanes have joined

        def backward_slice(i: int):
            lane = i % self.lanes
            g_out = dH[:, i * self.hs:(i + 1) * self.hs]  # CONCAT backward is a column view
            for l in reversed(range(self.L)):
                p, gr = self.params[i][l], self.grads[i][l]
                wi = self.widths[l][0]
                if l > 0:
                    g_in = self.dbuf[lane][l % 2][:, :wi]
                elif self.shared:  # the fused features are learned: the first slice writes, the others add
                    g_in = (self.dXin if i == 0 else self.dXs[i - 1] if deferred else self.dXtmp)[:, :wi]
                else:
                    g_in = None  # raw features need no gradient
                B.slicegcn_layer_bwd(self.g, self.hin(i, l), p["W_agg"], p["W_self"], self.zbuf(i, l), self.mask[i][l],
                                     g_out, g_in, gr["dW_agg"], gr["db"], gr["dW_self"], gr["db_self"], self.ws_lane[lane],
                                     act=self.act(l), order=self.order, layout=self.layout[l])
                if l == 0 and self.shared and i > 0 and not deferred:
                    B.slicegcn_accumulate(self.dXin[:, :wi], g_in)
                if fused and l == self.L - 1:  # dE[i] = column sums of dH^i = this layer's db_self
                    B.slicegcn_slice_feature(gr["db_self"].view(1, -1), 0, self.hs, self.dE[i].view(1, -1))
                g_out = g_in

        self._on_lanes(backward_slice)
        if deferred:
            for i in range(1, self.k):
                B.slicegcn_accumulate(self.dXin[:, :self.w0], self.dXs[i - 1][:, :self.w0])


class Classifier:
    """The paper's MLP_CLS on the concatenated representation followed by the mean softmax
    cross-entropy of its loss equation: logits = relu(H W1 + b1) W2 + b2.  Owns buffers and orders
    the library calls; every arithmetic step is a kernel of ``libslicegcn.so``."""

    def __init__(self, n_nodes: int, width: int, hidden: int, classes: int, device="cuda"):
        self.n, self.w, self.h, self.c = n_nodes, width, hidden, classes
        self.dev = torch.device(device)
        f32 = dict(dtype=torch.float32, device=self.dev)
        self.W1 = torch.zeros((width, hidden), **f32); self.b1 = torch.zeros(hidden, **f32)
        self.W2 = torch.zeros((hidden, classes), **f32); self.b2 = torch.zeros(classes, **f32)
        self.dW1 = torch.empty_like(self.W1); self.db1 = torch.empty_like(self.b1)
        self.dW2 = torch.empty_like(self.W2); self.db2 = torch.empty_like(self.b2)
        self.A = torch.empty((n_nodes, hidden), **f32)
        self.dA = torch.empty((n_nodes, hidden), **f32)
        self.mask = torch.zeros((n_nodes, (hidden + 31) // 32), dtype=torch.int32, device=self.dev)
        self.logits = torch.empty((n_nodes, classes), **f32)  # overwritten by its own gradient in backward
        self.loss = torch.zeros(1, **f32)
        ws = max(B.slicegcn_softmax_ce_workspace_bytes(n_nodes), B.slicegcn_linear_bwd_workspace_bytes(n_nodes, width, hidden),
                 B.slicegcn_linear_bwd_workspace_bytes(n_nodes, hidden, classes))
        self.ws = torch.empty(ws, dtype=torch.uint8, device=self.dev)

    def set_params(self, W1, b1, W2, b2):
        for dst, src in ((self.W1, W1), (self.b1, b1), (self.W2, W2), (self.b2, b2)):
            dst.copy_(src)

    def forward(self, H: torch.Tensor, labels: torch.Tensor) -> torch.Tensor:
        """Loss of the batch (device scalar).  Leaves the gradient of the loss with respect to the
        logits in ``self.logits`` for ``backward``."""
        B.slicegcn_linear_fwd(H, self.W1, self.b1, self.A, self.mask, act=B.ACT_RELU)
        B.slicegcn_linear_fwd(self.A, self.W2, self.b2, self.logits, None, act=B.ACT_NONE)
        B.slicegcn_softmax_ce(self.logits, labels, self.loss, self.logits, self.ws)  # gradient in place
        return self.loss

    def backward(self, H: torch.Tensor, dH: torch.Tensor):
        """dH receives the gradient of the loss with respect to H; the parameter gradients go to
        dW1, db1, dW2, db2."""
        B.slicegcn_linear_bwd(self.A, self.W2, None, self.logits, self.dA, self.dW2, self.db2, self.ws, act=B.ACT_NONE)
        B.slicegcn_linear_bwd(H, self.W1, self.mask, self.dA, dH, self.dW1, self.db1, self.ws, act=B.ACT_RELU)

    def forward_backward(self, H: torch.Tensor, labels: torch.Tensor, dH: torch.Tensor) -> torch.Tensor:
        self.forward(H, labels)
        self.backward(H, dH)
        return self.loss


class FeatureFusion:
    """The paper's MLP_FF (feature-fusion equation; two dense layers d' -> d' -> slice_size with a ReLU
    between them, shared by all slices): Xff = relu(X W1 + b1) W2 + b2.  Owns buffers and orders the
    library calls; every arithmetic step is a kernel of ``libslicegcn.so``."""

    def __init__(self, n_nodes: int, feat: int, out_width: int, device="cuda"):
        self.n, self.f, self.s = n_nodes, feat, out_width
        self.dev = torch.device(device)
        f32 = dict(dtype=torch.float32, device=self.dev)
        self.W1 = torch.zeros((feat, feat), **f32); self.b1 = torch.zeros(feat, **f32)
        self.W2 = torch.zeros((feat, out_width), **f32); self.b2 = torch.zeros(out_width, **f32)
        self.dW1 = torch.empty_like(self.W1); self.db1 = torch.empty_like(self.b1)
        self.dW2 = torch.empty_like(self.W2); self.db2 = torch.empty_like(self.b2)
        self.A = torch.empty((n_nodes, feat), **f32)
        self.dA = torch.empty((n_nodes, feat), **f32)
        self.mask = torch.zeros((n_nodes, (feat + 31) // 32), dtype=torch.int32, device=self.dev)
        self.Xff = torch.zeros((n_nodes, padded_ld(out_width)), **f32)  # padding columns stay zero
        ws = max(B.slicegcn_linear_bwd_workspace_bytes(n_nodes, feat, feat),
                 B.slicegcn_linear_bwd_workspace_bytes(n_nodes, feat, out_width))
        self.ws = torch.empty(ws, dtype=torch.uint8, device=self.dev)

    def set_params(self, W1, b1, W2, b2):
        for dst, src in ((self.W1, W1), (self.b1, b1), (self.W2, W2), (self.b2, b2)):
            dst.copy_(src)

    def forward(self, X: torch.Tensor) -> torch.Tensor:
        B.slicegcn_linear_fwd(X, self.W1, self.b1, self.A, self.mask, act=B.ACT_RELU)
        B.slicegcn_linear_fwd(self.A, self.W2, self.b2, self.Xff[:, :self.s], None, act=B.ACT_NONE)
        return self.Xff

    def backward(self, X: torch.Tensor, dXff: torch.Tensor):
        """dXff: n x out_width gradient of the fused features (the sum over the slice models)."""
        B.slicegcn_linear_bwd(self.A, self.W2, None, dXff, self.dA, self.dW2, self.db2, self.ws, act=B.ACT_NONE)
        B.slicegcn_linear_bwd(X, self.W1, self.mask, self.dA, None, self.dW1, self.db1, self.ws, act=B.ACT_RELU)


def _dense_slots(obj):
    return [(obj, "W1", obj, "dW1"), (obj, "b1", obj, "db1"), (obj, "W2", obj, "dW2"), (obj, "b2", obj, "db2")]


Classifier.parameter_slots = _dense_slots
FeatureFusion.parameter_slots = _dense_slots


class Optimizer:
    """Adam with a cosine-annealed learning rate (the paper's experimental settings) over all learnable
    tensors of the given models.  The tensors are moved into one flat buffer (gradients into another) and
    the models' attributes rebound to views of it, so one library call updates every parameter."""

    ALIGN = 64  # floats: every tensor starts on a 256-byte boundary, so vector paths stay usable

    def __init__(self, models, lr_max: float, lr_min: float = 0.0, t_max: int = 1, beta1: float = 0.9,
                 beta2: float = 0.999, eps: float = 1e-8, weight_decay: float = 0.0):
        slots = [s for m in models for s in m.parameter_slots()]
        get = lambda o, k: o[k] if isinstance(o, dict) else getattr(o, k)
        offs, total = [], 0
        for po, pk, _, _ in slots:
            offs.append(total)
            total += (get(po, pk).numel() + self.ALIGN - 1) // self.ALIGN * self.ALIGN
        dev = get(slots[0][0], slots[0][1]).device
        self.P, self.G, self.M, self.V = (torch.zeros(total, dtype=torch.float32, device=dev) for _ in range(4))
        for (po, pk, go, gk), o in zip(slots, offs):
            old = get(po, pk)
            pv = self.P[o:o + old.numel()].view(old.shape)
            pv.copy_(old)
            gv = self.G[o:o + old.numel()].view(old.shape)
            for holder, key, view in ((po, pk, pv), (go, gk, gv)):
                if isinstance(holder, dict):
                    holder[key] = view
                else:
                    setattr(holder, key, view)
        self.hyper = (beta1, beta2, eps, weight_decay)
        self.lr_max, self.lr_min, self.t_max = lr_max, lr_min, t_max
        self.t = 0

    def step(self, epoch: int) -> float:
        """One update with the learning rate of ``epoch`` (0-based); returns that rate."""
        self.t += 1
        lr = B.slicegcn_cosine_lr(self.lr_max, self.lr_min, epoch, self.t_max)
        b1, b2, eps, wd = self.hyper
        B.slicegcn_adam_step(self.P, self.G, self.M, self.V, lr, self.t, b1, b2, eps, wd)
        return lr


class GraphedStep:
    """A sequence of library calls captured once into a HIP graph and replayed with one launch.

    For the small workloads a pass is a few hundred kernels of microseconds each and the time goes
    into launching them; a replayed graph removes that.  ``fn`` must only issue library calls on the
    current stream and touch preallocated buffers (every entry point except graph construction
    qualifies: none allocates, synchronises or clears memory with a memset node).  The buffers are
    read through their addresses, so new inputs written into the same tensors are picked up by the
    next replay."""

    def __init__(self, fn, warmup: int = 1):
        self.stream = torch.cuda.Stream()
        self.stream.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(self.stream):
            for _ in range(warmup):
                fn()
        torch.cuda.current_stream().wait_stream(self.stream)
        torch.cuda.synchronize()
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph, stream=self.stream):
            fn()

    def replay(self):
        self.graph.replay()
