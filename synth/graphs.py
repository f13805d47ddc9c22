"""Seeded synthetic graphs: G(n, M) Erdos-Renyi, R-MAT and planted-community edge lists.

Both return ``M_und`` distinct undirected edges (u != v) as two int64 tensors
(src, dst), in order of first occurrence in the counter-indexed stream of draws, so the
result does not depend on how the draws were batched.  Vertices are then relabelled by a
seeded random permutation (hubs land anywhere in the index range).

Inputs only: nothing here normalises, aggregates or otherwise touches the GCN method.
"""
from __future__ import annotations

import math

import torch

from . import rng

STREAM_EDGES = 0
STREAM_PERM = 1


def _first_distinct(draw_fn, n_nodes: int, m_und: int, device, batch: int):
    """First ``m_und`` distinct valid undirected pairs of the indexed draw stream.

    ``draw_fn(idx)`` maps an int64 index tensor to (u, v) endpoint tensors.  A draw is
    valid when both endpoints are < n_nodes and differ.  Returns (lo, hi) with lo < hi.
    """
    keys = torch.empty(0, dtype=torch.int64, device=device)  # distinct keys so far
    first = torch.empty(0, dtype=torch.int64, device=device)  # their first draw index
    cursor = 0
    rounds = 0
    while keys.numel() < m_und:
        rounds += 1
        if rounds > 400:
            raise RuntimeError("edge generator: too many rounds (graph too dense for this recipe)")
        idx = rng.arange64(batch, device, cursor)
        cursor += batch
        u, v = draw_fn(idx)
        ok = (u < n_nodes) & (v < n_nodes) & (u != v)
        u, v, idx = u[ok], v[ok], idx[ok]
        k_new = torch.minimum(u, v) * n_nodes + torch.maximum(u, v)
        all_k = torch.cat([keys, k_new])
        all_i = torch.cat([first, idx])
        uniq, inv = torch.unique(all_k, return_inverse=True)
        fmin = torch.full((uniq.numel(),), torch.iinfo(torch.int64).max, dtype=torch.int64, device=device)
        fmin.scatter_reduce_(0, inv, all_i, reduce="amin")
        keys, first = uniq, fmin
    # keep the m_und keys that appeared earliest, in order of appearance
    order = torch.argsort(first)[:m_und]
    # every key whose first index is below the cut is in the set, whatever the batching was
    keys = keys[order]
    return keys // n_nodes, keys % n_nodes


def _permute(lo, hi, n_nodes: int, seed: int):
    dev = lo.device
    perm = torch.argsort(rng.bits(seed, STREAM_PERM, rng.arange64(n_nodes, dev)), stable=True)
    return perm[lo], perm[hi]


def erdos_renyi(n_nodes: int, m_und: int, seed: int, device="cpu", permute: bool = True):
    """G(n, M): uniform endpoint pairs until m_und distinct undirected edges exist."""
    if m_und > n_nodes * (n_nodes - 1) // 2:
        raise ValueError("m_und exceeds the number of vertex pairs")

    def draw(idx):
        u = (rng.uniform(seed, STREAM_EDGES, 2 * idx) * n_nodes).to(torch.int64)
        v = (rng.uniform(seed, STREAM_EDGES, 2 * idx + 1) * n_nodes).to(torch.int64)
        return u, v

    lo, hi = _first_distinct(draw, n_nodes, m_und, device, batch=max(1024, int(m_und * 1.25)))
    return _permute(lo, hi, n_nodes, seed) if permute else (lo, hi)


def rmat(n_nodes: int, m_und: int, seed: int, a=0.57, b=0.19, c=0.19, d=0.05,
         device="cpu", permute: bool = True, batch: int | None = None):
    """R-MAT: one quadrant draw per bit level, scale = ceil(log2 n_nodes), no noise."""
    if abs(a + b + c + d - 1.0) > 1e-12:
        raise ValueError("quadrant probabilities must sum to 1")
    scale = max(1, math.ceil(math.log2(n_nodes)))

    def draw(idx):
        u = torch.zeros_like(idx)
        v = torch.zeros_like(idx)
        for level in range(scale):
            r = rng.uniform(seed, STREAM_EDGES, idx * scale + level)
            ubit = (r >= a + b).to(torch.int64)                     # quadrants c, d: lower half
            vbit = ((r >= a) & (r < a + b) | (r >= a + b + c)).to(torch.int64)  # quadrants b, d
            u = (u << 1) | ubit
            v = (v << 1) | vbit
        return u, v

    if batch is None:
        batch = max(1024, min(int(m_und * 1.3), 1 << 26))
    lo, hi = _first_distinct(draw, n_nodes, m_und, device, batch=batch)
    return _permute(lo, hi, n_nodes, seed) if permute else (lo, hi)


def planted_communities(n_nodes: int, community: int, d_in: int, d_out: int, seed: int, device="cpu", permute: bool = True):
    """Planted communities (a stochastic block model with equal blocks): vertex v of block v // community
    draws ``d_in`` neighbours uniformly inside its block and ``d_out`` uniformly over the whole graph.  Returns
    the n_nodes * (d_in + d_out) drawn pairs as they come (repeats and self pairs included: the adjacency
    builder collapses them), so the number of distinct edges is a little below that.  With ``permute`` the
    vertices are relabelled by a seeded random permutation: the communities are then scattered over the index
    range, which is the situation a locality-restoring row order has to undo.  (R-MAT has no such structure.)"""
    per = d_in + d_out
    idx = rng.arange64(n_nodes * per, device)
    v = idx // per
    j = idx % per
    block = v // community
    size = torch.clamp(n_nodes - block * community, max=community)   # the last block may be short
    u_in = block * community + (rng.uniform(seed, STREAM_EDGES, idx) * size).to(torch.int64)
    u_out = (rng.uniform(seed, STREAM_EDGES, idx) * n_nodes).to(torch.int64)
    u = torch.where(j < d_in, u_in, u_out)
    return _permute(v, u, n_nodes, seed) if permute else (v, u)
