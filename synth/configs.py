"""The five benchmark workloads and their seeded tensors.

Shapes follow the paper's node-classification datasets (its dataset-statistics table gives
the citation-graph shape used by ``cfg2``); the graphs and features themselves are synthetic.
Per-slice hidden width is total hidden / k, the paper's "scale each layer down by p" rule.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import torch

from . import graphs, rng

BASE_SEED = 240811500
STREAM_X, STREAM_W, STREAM_LABELS, STREAM_DH, STREAM_E = 2, 3, 4, 5, 6


@dataclass(frozen=True)
class Workload:
    name: str
    cfg_id: int
    n_nodes: int
    m_und: int          # distinct undirected off-diagonal edges
    feat: int           # F
    k: int              # number of slices
    hidden: int         # total hidden width H (per slice: H // k)
    layers: int
    classes: int
    kind: str           # "er" | "rmat" | "comm" (planted communities: m_und is then an upper bound)

    @property
    def seed(self) -> int:
        return BASE_SEED + self.cfg_id

    @property
    def nnz(self) -> int:
        return 2 * self.m_und + self.n_nodes

    @property
    def slice_width(self) -> int:
        return -(-self.feat // self.k)

    @property
    def slice_hidden(self) -> int:
        return self.hidden // self.k


COMM_SIZE, COMM_D_IN, COMM_D_OUT = 512, 24, 2

WORKLOADS = {
    "cfg1": Workload("cfg1", 1, 2_048, 4_096, 128, 2, 64, 2, 8, "er"),
    "cfg2": Workload("cfg2", 2, 169_343, 1_185_401, 128, 4, 256, 3, 40, "rmat"),
    "cfg3": Workload("cfg3", 3, 232_965, 57_000_000, 602, 2, 256, 2, 41, "rmat"),
    "cfg4": Workload("cfg4", 4, 2_449_029, 62_000_000, 100, 4, 256, 3, 47, "rmat"),
    "cfg5": Workload("cfg5", 5, 10_000_000, 150_000_000, 256, 8, 256, 3, 64, "rmat"),
    # not one of the five benchmark workloads: 2 M nodes in planted communities of 512, scattered over the index
    # range by the random relabelling -- the input on which a locality-restoring row order can be measured
    "comm": Workload("comm", 6, 2_000_000, 2_000_000 * (COMM_D_IN + COMM_D_OUT), 128, 4, 128, 2, 16, "comm"),
}


def get_workload(name: str) -> Workload:
    """A named workload, or ``er:<n_nodes>:<m_und>``: a uniform random graph with one 32-wide slice (used to
    measure what the aggregation's row gathers cost as a function of the size of the gathered matrix)."""
    if name.startswith("er:"):
        _, n, m = name.split(":")
        return Workload(name, 100, int(n), int(m), 32, 1, 32, 1, 2, "er")
    return WORKLOADS[name]


def edges(w: Workload, device="cpu", permute: bool = True):
    if w.kind == "er":
        return graphs.erdos_renyi(w.n_nodes, w.m_und, w.seed, device=device, permute=permute)
    if w.kind == "comm":
        return graphs.planted_communities(w.n_nodes, COMM_SIZE, COMM_D_IN, COMM_D_OUT, w.seed, device=device, permute=permute)
    return graphs.rmat(w.n_nodes, w.m_und, w.seed, device=device, permute=permute)


def normal_matrix(seed: int, stream: int, rows: int, cols: int, device="cpu", std: float = 1.0,
                  col_start: int = 0, col_count: int | None = None, ld: int | None = None,
                  row_chunk: int = 1 << 20) -> torch.Tensor:
    """fp32 N(0, std^2) matrix; element (i, j) depends only on (seed, stream, i*cols + j).

    ``col_start/col_count`` produce a column block of the logical rows x cols matrix without
    materialising the rest; ``ld`` pads each row with zeros to that leading dimension.
    """
    cc = cols - col_start if col_count is None else col_count
    ld = cc if ld is None else ld
    out = torch.zeros((rows, ld), dtype=torch.float32, device=device)
    j = rng.arange64(cc, device, col_start)
    for r0 in range(0, rows, row_chunk):
        r1 = min(rows, r0 + row_chunk)
        idx = rng.arange64(r1 - r0, device, r0)[:, None] * cols + j[None, :]
        out[r0:r1, :cc] = (rng.normal(seed, stream, idx) * std).to(torch.float32)
    return out


def features(w: Workload, device="cpu", **kw) -> torch.Tensor:
    return normal_matrix(w.seed, STREAM_X, w.n_nodes, w.feat, device=device, **kw)


def glorot(seed: int, tag: int, fan_in: int, fan_out: int, device="cpu") -> torch.Tensor:
    """fp32 Glorot-uniform fan_in x fan_out matrix; ``tag`` separates the matrices of a model."""
    lim = math.sqrt(6.0 / (fan_in + fan_out))
    idx = rng.arange64(fan_in * fan_out, device) + (tag << 32)
    u = rng.uniform(seed, STREAM_W, idx)
    return ((2.0 * u - 1.0) * lim).to(torch.float32).reshape(fan_in, fan_out)


def labels(w: Workload, device="cpu") -> torch.Tensor:
    u = rng.uniform(w.seed, STREAM_LABELS, rng.arange64(w.n_nodes, device))
    return (u * w.classes).to(torch.int64)
