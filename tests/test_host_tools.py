"""Host-side checks of the benchmark driver and the synthetic inputs that need no GPU: the command-line contract of
bench.py, the algorithmic-byte formula it reports, and the determinism and shape of the seeded generators."""
import os
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_algorithmic_bytes_formula():
    import bench
    # 4 B index + 4 B value per stored entry, row pointers, every operand row read once and every output row written once
    n, nnz, w = 10_000_000, 310_000_000, 32
    assert bench.spmm_bytes(n, nnz, w) == 8 * nnz + 4 * (n + 1) + 8 * n * w == 5_080_000_004


def test_workloads_match_the_stated_sizes():
    import synth
    want = {"cfg1": (2048, 10_240, 128, 2), "cfg2": (169_343, 2_540_145, 128, 4), "cfg3": (232_965, 114_232_965, 602, 2),
            "cfg4": (2_449_029, 126_449_029, 100, 4), "cfg5": (10_000_000, 310_000_000, 256, 8)}
    for name, (n, nnz, feat, k) in want.items():
        w = synth.WORKLOADS[name]
        assert (w.n_nodes, w.nnz, w.feat, w.k) == (n, nnz, feat, k)
        assert w.nnz == 2 * w.m_und + w.n_nodes


def test_generators_are_seeded_and_chunk_independent():
    from synth import configs
    w = configs.get_workload("cfg1")
    s1, d1 = configs.edges(w)
    s2, d2 = configs.edges(w)
    assert np.array_equal(s1.numpy(), s2.numpy()) and np.array_equal(d1.numpy(), d2.numpy())
    assert s1.numel() == w.m_und and int((s1 == d1).sum()) == 0
    und = {(min(a, b), max(a, b)) for a, b in zip(s1.tolist(), d1.tolist())}
    assert len(und) == w.m_und                      # distinct undirected edges
    X = configs.features(w)
    block = configs.features(w, col_start=64, col_count=64)     # a column block without materialising the rest
    assert np.array_equal(X[:, 64:128].numpy(), block.numpy())
    chunked = configs.normal_matrix(w.seed, configs.STREAM_X, w.n_nodes, w.feat, row_chunk=100)
    assert np.array_equal(X.numpy(), chunked.numpy())
    assert abs(float(X.mean())) < 0.01 and abs(float(X.std()) - 1.0) < 0.01


def test_planted_communities_and_uniform_graphs():
    from synth import configs, graphs
    s, d = graphs.planted_communities(4096, 128, 12, 1, seed=5, device="cpu", permute=False)
    same = (s // 128) == (d // 128)
    assert 0.85 < float(same.float().mean()) < 0.97     # 12 of 13 draws stay inside the community
    w = configs.get_workload("er:1000:8000")
    assert (w.n_nodes, w.m_und, w.k, w.feat) == (1000, 8000, 1, 32)
    s, d = configs.edges(w)
    assert s.numel() == 8000 and int(s.max()) < 1000 and int(d.max()) < 1000
