"""Parity at the benchmark's full size (cfg5: 10M nodes, 310M stored entries, slices of 32), in
the launch configuration bench.py times.  The oracle builds its own CSR from the same edge list
on the host (bit-exact comparison of the whole structure), and the aggregation is compared on
sampled output rows the oracle computes one by one, plus the fixed-point invariant
A^ (D~^1/2 1) = D~^1/2 1, which holds at any size.
"""
import numpy as np
import pytest
import torch

import oracle
import synth
from synth import configs
import paper_2408_11500_amd as sg
from paper_2408_11500_amd.stack import padded_ld
from gpu_util import TOL, rel_err

pytestmark = pytest.mark.gpu


def _run(name: str, n_samples: int):
    w = synth.WORKLOADS[name]
    dev = torch.device("cuda")
    print(f"[fullsize] {name}: generating", flush=True)
    src, dst = configs.edges(w, device=dev)
    g = sg.slicegcn_build_norm_csr(src, dst, w.n_nodes)
    print(f"[fullsize] {name}: oracle CSR build on the host", flush=True)
    o = oracle.build_norm_csr(src.cpu().numpy(), dst.cpu().numpy(), w.n_nodes)
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
    print(f"[fullsize] {name}: {rows.size} sampled rows, max rel err {err:.2e}, max degree {int(o.deg.max())}", flush=True)
    assert err <= TOL
    bound = oracle.spmm_rows(o, np.abs(X64), rows) * TOL
    assert np.all(np.abs(got - want) <= bound + 1e-30)
    # bitwise reproducible
    Y2 = torch.empty_like(Y)
    sg.slicegcn_spmm_slice(g, Xs[:, :width], Y2[:, :width])
    assert torch.equal(Y[:, :width], Y2[:, :width])
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
    g.destroy()


def test_cfg4_full_size_sampled():
    _run("cfg4", 2000)


def test_cfg5_full_size_sampled():
    _run("cfg5", 2000)
