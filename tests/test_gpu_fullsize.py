"""Parity at the full size of the three large workloads (cfg3, cfg4, cfg5), in the launch configuration
bench.py times.  The oracle builds its own CSR from the same edge list on the host (bit-exact comparison
of the whole structure); the aggregation is compared on sampled output rows the oracle computes one by
one, plus the fixed-point invariant A^ (D~^1/2 1) = D~^1/2 1, which holds at any size; the adjoint identity <A^ X, G> = <X, A^ G> over every row with random operands; and a chain of two
layers of one slice runs forward and backward with every output element compared with the oracle.
"""
import numpy as np
import pytest
import torch

import oracle
import synth
from synth import configs
import paper_2408_11500_amd as sg
from paper_2408_11500_amd.stack import padded_ld
from gpu_util import TOL, progress, rel_err

pytestmark = pytest.mark.gpu



_CACHE = {}


def _graph(name: str):
    """(workload, handle, oracle CSR) of a workload, built once per test session and shared by its tests."""
    if name not in _CACHE:
        for other in list(_CACHE):       # one large workload at a time
            _CACHE.pop(other)[1].destroy()
        w = synth.WORKLOADS[name]
        dev = torch.device("cuda")
        progress(f"[fullsize] {name}: generating")
        src, dst = configs.edges(w, device=dev)
        g = sg.slicegcn_build_norm_csr(src, dst, w.n_nodes)
        progress(f"[fullsize] {name}: oracle CSR build on the host")
        o = oracle.build_norm_csr(src.cpu().numpy(), dst.cpu().numpy(), w.n_nodes)
        _CACHE[name] = (w, g, o)
    return _CACHE[name]


def _run(name: str, n_samples: int):
    w, g, o = _graph(name)
    dev = torch.device("cuda")
    assert o.nnz == w.nnz
    h = g.to_host()
    assert np.array_equal(h["rowptr"].astype(np.int64), o.rowptr)
    assert np.array_equal(h["colidx"], o.colidx)
    assert np.array_equal(h["deg"], o.deg)
    assert np.max(np.abs(h["dinv"] / o.dinv - 1.0)) <= 1e-6
    assert np.max(np.abs(h["vals"] / o.vals - 1.0)) <= 1e-6
    del h

    slices, width = sg.slicegcn_slice_strategy(w.feat, w.k)
    a, b = slices[w.k - 1]                                   # last slice: non-zero column offset
    ld = padded_ld(width)
    Xs = configs.features(w, device=dev, col_start=a, col_count=b - a, ld=ld)
    Y = torch.empty((w.n_nodes, ld), dtype=torch.float32, device=dev)
    sg.slicegcn_spmm_slice(g, Xs[:, :width], Y[:, :width])
    # sampled rows: the longest rows (cut into segments), shortest rows, and random ones
    rng = np.random.default_rng(w.seed)
    order = np.argsort(o.deg)
    rows = np.unique(np.concatenate([order[-40:], order[:40], rng.integers(0, w.n_nodes, n_samples)]))
    X64 = Xs[:, :width].cpu().numpy().astype(np.float64)
    want = oracle.spmm_rows(o, X64, rows)
    got = Y[:, :width][torch.as_tensor(rows, device=dev)].cpu().numpy()
    scale = float(np.max(np.abs(want)))
    err = float(np.max(np.abs(got - want))) / scale
    progress(f"[fullsize] {name}: {rows.size} sampled rows, max rel err {err:.2e}, max degree {int(o.deg.max())}")
    assert err <= TOL
    bound = oracle.spmm_rows(o, np.abs(X64), rows) * TOL
    assert np.all(np.abs(got - want) <= bound + 1e-30)
    # bitwise reproducible
    Y2 = torch.empty_like(Y)
    sg.slicegcn_spmm_slice(g, Xs[:, :width], Y2[:, :width])
    assert torch.equal(Y[:, :width], Y2[:, :width])
    # the factored form (operand rows carry D~^-1/2, the stored values are not read): what the default step of
    # bench.py runs at this size.  Same rows, same oracle values.
    sg.slicegcn_scale_rows(g, Xs[:, :width], Y2[:, :width])
    sg.slicegcn_spmm_slice(g, Y2[:, :width], Y[:, :width], prescaled=True)
    got = Y[:, :width][torch.as_tensor(rows, device=dev)].cpu().numpy()
    err = float(np.max(np.abs(got - want))) / scale
    progress(f"[fullsize] {name}: factored form, max rel err {err:.2e}")
    assert err <= TOL
    assert np.all(np.abs(got - want) <= bound + 1e-30)
    # invariant at full size: every row, no sampling
    s = torch.as_tensor(np.sqrt(o.deg.astype(np.float64)), dtype=torch.float32, device=dev)
    S = torch.zeros((w.n_nodes, 32), dtype=torch.float32, device=dev)
    S[:, 0] = s
    S[:, 5] = -2.0 * s
    R = torch.empty_like(S)
    sg.slicegcn_spmm_slice(g, S, R)
    assert float(torch.max(torch.abs(R[:, 0] / s - 1.0))) <= TOL
    assert float(torch.max(torch.abs(R[:, 5] / (-2.0 * s) - 1.0))) <= TOL
    assert float(torch.max(torch.abs(R[:, 1]))) == 0.0
    # adjoint identity at full size, every row with random signs: <A^ X, G> = <X, A^T G>, the right side through the
    # transposed call.  Inner products in fp64 over the fp32 results: the two sides differ by the rounding of the
    # n * w output elements (random signs: about 1e-7 / sqrt(n w) of |A^X| |G|, some 1e-11), whereas one output row
    # dropped, doubled or written to the wrong place in either call shifts a side by about 1 / (n sqrt(w)) of it
    # (2e-8 at 10 M rows x 32 columns)
    G = configs.normal_matrix(w.seed, configs.STREAM_DH, w.n_nodes, ld, device=dev)
    sg.slicegcn_spmm_slice(g, Xs[:, :width], Y[:, :width])
    lhs = float((Y[:, :width].double() * G[:, :width].double()).sum())
    sg.slicegcn_spmm_slice(g, G[:, :width], Y2[:, :width], transpose=True)
    rhs = float((Xs[:, :width].double() * Y2[:, :width].double()).sum())
    norm = float(Y[:, :width].double().norm() * G[:, :width].double().norm())
    progress(f"[fullsize] {name}: adjoint identity, |lhs - rhs| / (|A^X| |G|) = {abs(lhs - rhs) / norm:.2e}")
    assert abs(lhs - rhs) <= 2e-9 * norm


def _layer_chain(name: str, slice_id: int, n_layers: int = 2):
    """Layers 1 and 2 of one slice at the workload's real size (its slice width -> per-slice hidden ->
    per-slice hidden), forward then backward (the second layer with its input gradient, the first without, as
    in a pass over raw features), every output element against the oracle.  The backward pass differentiates
    the oracle's activation patterns on both sides.  With ``n_layers`` = 1 only the first layer runs, with its
    input gradient (as under feature fusion).

    The layers run in the layout the stack (and so bench.py) uses at these sizes: activations that feed an
    aggregation are kept as D~^-1/2 H (raw slice scaled once, every layer but the last stores scaled); the
    oracle works on the unscaled tensors, and what the library reads or writes scaled is compared through the
    oracle's own D~^-1/2."""
    from synth import model
    from gpu_util import assert_close, pack_mask, unpack_mask
    w, g, o = _graph(name)
    dev = torch.device("cuda")
    n, hs = w.n_nodes, w.slice_hidden
    slices, width = sg.slicegcn_slice_strategy(w.feat, w.k)
    a, b = slices[slice_id]
    f32 = dict(dtype=torch.float32, device=dev)
    shapes = [(width, hs), (hs, hs)][:n_layers]
    Xs = configs.features(w, device=dev, col_start=a, col_count=b - a, ld=padded_ld(width))
    sg.slicegcn_scale_rows(g, Xs[:, :width], Xs[:, :width])        # in place, once: the raw features are constant
    IN, OUT = sg.binding.LAYER_IN_SCALED, sg.binding.LAYER_OUT_SCALED
    layout = [IN | (OUT if l < n_layers - 1 else 0) for l in range(n_layers)]
    dinv = o.dinv[:, None]
    params = [model.slice_layer_params(w, slice_id, l, wi, wo, bias_std=0.05) for l, (wi, wo) in enumerate(shapes)]
    H = [Xs[:, :width], torch.empty((n, padded_ld(hs)), **f32)[:, :hs], torch.empty((n, hs), **f32)][:n_layers + 1]
    Z = [torch.empty((n, padded_ld(wi)), **f32)[:, :wi] for wi, _ in shapes]
    mask = [torch.zeros((n, (wo + 31) // 32), dtype=torch.int32, device=dev) for _, wo in shapes]
    for l in range(n_layers):
        Wa, bb, Ws, bs = (t.cuda() for t in params[l])
        sg.slicegcn_layer_fwd(g, H[l], Wa, bb, Ws, bs, H[l + 1], Z[l], mask[l], layout=layout[l])
    progress(f"[fullsize-layer] {name}: oracle forward")
    h64 = Xs[:, :width].cpu().numpy().astype(np.float64) / dinv      # the unscaled input the scaled fp32 rows stand for
    saved = []
    for l in range(n_layers):
        Wa, bb, Ws, bs = (t.numpy() for t in params[l])
        hin = h64
        h64, Zo, Po = oracle.layer_fwd(o, hin, Wa, bb, Ws, bs, act=1)
        e1 = assert_close(Z[l].cpu().numpy(), Zo, f"Z of layer {l + 1}")
        e2 = assert_close(H[l + 1].cpu().numpy(), dinv * h64 if layout[l] & OUT else h64, f"output of layer {l + 1}")
        ref_mask = Po > 0
        differ = unpack_mask(mask[l].cpu().numpy(), shapes[l][1]) != ref_mask
        assert np.all(np.abs(Po[differ]) <= 1e-5 * np.sqrt(np.mean(Po * Po)))
        progress(f"[fullsize-layer] {name}: layer {l + 1} forward ok (Z {e1:.1e}, out {e2:.1e}), {int(differ.sum())} "
                 f"activation decisions inside the rounding band")
        mask[l].copy_(torch.as_tensor(pack_mask(ref_mask.astype(np.uint8))))
        saved.append((hin, Zo, ref_mask))
        del Po
    # backward: layer 2 (with input gradient), then layer 1 (without)
    dH = configs.normal_matrix(w.seed, configs.STREAM_DH, n, hs, device=dev)
    g_out, ref_out = dH, dH.cpu().numpy().astype(np.float64)
    for l in reversed(range(n_layers)):
        wi, wo = shapes[l]
        Wa, bb, Ws, bs = (t.cuda() for t in params[l])
        need = l > 0 or n_layers == 1
        dHin = torch.empty((n, padded_ld(wi)), **f32)[:, :wi] if need else None
        dW_agg = torch.empty((wi, wo), **f32); db = torch.empty(wo, **f32)
        dW_self = torch.empty((wi, wo), **f32); db_self = torch.empty(wo, **f32)
        ws = torch.empty(sg.slicegcn_layer_bwd_workspace_bytes(g, wi, wo, need), dtype=torch.uint8, device=dev)
        sg.slicegcn_layer_bwd(g, H[l], Wa, Ws, Z[l], mask[l], g_out, dHin, dW_agg, db, dW_self, db_self, ws, layout=layout[l])
        progress(f"[fullsize-layer] {name}: oracle backward of layer {l + 1}")
        hin, Zo, ref_mask = saved[l]
        ref = oracle.layer_bwd(o, hin, Zo, ref_mask, params[l][0].numpy(), params[l][2].numpy(), ref_out, need_dHin=need)
        outs = [("dW_agg", dW_agg), ("db", db), ("dW_self", dW_self), ("db_self", db_self)] + ([("dHin", dHin)] if need else [])
        for nm, t in outs:
            e = assert_close(t.cpu().numpy(), ref[nm], f"{nm} of layer {l + 1}")
            progress(f"[fullsize-layer] {name}: layer {l + 1} {nm}: max rel err {e:.2e}")
        if need:
            g_out, ref_out = dHin, ref["dHin"]
        del ws


def test_cfg3_full_size_sampled():
    _run("cfg3", 500)      # slices of 301 columns: three column passes, rows of up to 10^5 entries


def test_cfg3_full_size_layer_chain():
    _layer_chain("cfg3", 1)     # 301 -> 128 -> 128 on 233 K rows: the staged dense kernel and 1024-row gradient blocks


def test_cfg4_full_size_sampled():
    _run("cfg4", 2000)


def test_cfg4_full_size_layer_chain():
    _layer_chain("cfg4", 2)     # 25 -> 64 -> 64 on 2.4 M rows: the 64-wide strip kernels


def test_cfg5_full_size_sampled():
    _run("cfg5", 2000)


def test_cfg5_full_size_layer_chain():
    _layer_chain("cfg5", 1)     # 32 -> 32 -> 32 on 10 M rows: the 32-wide strip kernels, scaled output of layer 1 into layer 2


def test_release_cached_graphs():
    for name in list(_CACHE):
        _CACHE.pop(name)[1].destroy()
