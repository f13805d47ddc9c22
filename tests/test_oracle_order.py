"""Pins of the oracle's row orders (the optional locality preprocessing): hand-worked graphs, the
invariants of a first-in-first-out traversal, and scipy's breadth-first order on connected graphs."""
import numpy as np
import pytest
import scipy.sparse as sp
from scipy.sparse.csgraph import breadth_first_order, connected_components

import oracle


def _graph(edges, n, flags=3):
    e = np.asarray(edges, dtype=np.int64).reshape(-1, 2)
    return oracle.build_norm_csr(e[:, 0], e[:, 1], n, flags)


def test_degree_order_hand_example():
    # stored entries per row (self loop included): 0:2  1:4  2:4  3:3  4:2  5:1
    g = _graph([(0, 1), (1, 2), (1, 3), (2, 3), (2, 4)], 6)
    assert g.deg.tolist() == [2, 4, 4, 3, 2, 1]
    assert oracle.row_order(g, oracle.ORDER_DEGREE).tolist() == [1, 2, 3, 0, 4, 5]   # ties by ascending id


def test_bfs_order_hand_examples():
    # path 0-1-2-3-4: the first row of largest degree is 1; its neighbours 0 and 2 follow in ascending id, then 3, 4
    path = _graph([(i, i + 1) for i in range(4)], 5)
    assert oracle.row_order(path, oracle.ORDER_BFS).tolist() == [1, 0, 2, 3, 4]
    # star with centre 3: the centre, then the leaves in ascending id
    star = _graph([(3, j) for j in range(7) if j != 3], 7)
    assert oracle.row_order(star, oracle.ORDER_BFS).tolist() == [3, 0, 1, 2, 4, 5, 6]
    # two components and an isolated row: the triangle-with-tail first (root 2, degree 4), then the pair, then 7
    g = _graph([(0, 1), (1, 2), (0, 2), (2, 3), (5, 6)], 8)
    assert oracle.row_order(g, oracle.ORDER_BFS).tolist() == [2, 0, 1, 3, 5, 6, 4, 7]
    # with one tree only, the rows of the other components follow in degree order (5, 6 before 4, 7)
    assert oracle.row_order(g, oracle.ORDER_BFS, max_trees=1).tolist() == [2, 0, 1, 3, 5, 6, 4, 7]
    # a complete binary tree of depth 3 rooted anywhere: root = first row of degree 4 (an inner node: id 1)
    tree = _graph([(i, 2 * i + 1) for i in range(3)] + [(i, 2 * i + 2) for i in range(3)], 7)
    assert oracle.row_order(tree, oracle.ORDER_BFS).tolist() == [1, 0, 3, 4, 2, 5, 6]


@pytest.mark.parametrize("seed", range(6))
def test_bfs_order_invariants_and_scipy(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(20, 400))
    m = int(rng.integers(n // 2, 3 * n))
    g = _graph(np.stack([rng.integers(0, n, m), rng.integers(0, n, m)], 1), n)
    for mode in (oracle.ORDER_DEGREE, oracle.ORDER_BFS):
        order = oracle.row_order(g, mode)
        assert sorted(order.tolist()) == list(range(n))                         # a permutation
    by_deg = oracle.row_order(g, oracle.ORDER_DEGREE)
    d = g.deg[by_deg]
    assert np.all(d[:-1] >= d[1:]) and np.all((d[:-1] > d[1:]) | (by_deg[:-1] < by_deg[1:]))
    order = oracle.row_order(g, oracle.ORDER_BFS, max_trees=n)                  # every component gets its own tree
    pos = np.empty(n, dtype=np.int64); pos[order] = np.arange(n)
    A = sp.csr_matrix((np.ones(g.nnz), g.colidx, g.rowptr), shape=(n, n))
    ncomp, label = connected_components(A, directed=False)
    # each component is one contiguous run, and inside it the order is scipy's breadth-first order from the
    # run's first row (scipy also visits the neighbours of a row in index order)
    p = 0
    seen = set()
    while p < n:
        root = int(order[p])
        comp = label[root]
        assert comp not in seen
        seen.add(comp)
        size = int(np.sum(label == comp))
        run = order[p:p + size]
        assert np.all(label[run] == comp)
        ref, _ = breadth_first_order(A, root, directed=False, return_predecessors=True)
        assert run.tolist() == ref.tolist()
        # the root is the row of largest degree among everything not placed before it (ties: smallest id)
        rest = order[p:]
        best = max(g.deg[rest])
        assert g.deg[root] == best and root == min(int(v) for v in rest if g.deg[v] == best)
        p += size
    assert len(seen) == ncomp
    # queue invariant: the earliest-placed neighbour ("parent") positions never decrease along a tree
    parent_pos = np.array([min(pos[u] for u in g.colidx[g.rowptr[v]:g.rowptr[v + 1]]) for v in order])
    assert np.all(parent_pos <= np.arange(n))


def test_bfs_tree_limit_falls_back_to_degree_order():
    rng = np.random.default_rng(9)
    n = 300
    g = _graph(np.stack([rng.integers(0, 60, 200), rng.integers(0, 60, 200)], 1), n)   # rows 60.. are isolated
    order = oracle.row_order(g, oracle.ORDER_BFS, max_trees=2)
    full = oracle.row_order(g, oracle.ORDER_BFS, max_trees=n)
    by_deg = oracle.row_order(g, oracle.ORDER_DEGREE)
    # the first two trees agree with the unlimited traversal; the tail is the degree order of what is left
    A = sp.csr_matrix((np.ones(g.nnz), g.colidx, g.rowptr), shape=(n, n))
    _, label = connected_components(A, directed=False)
    k = int(np.sum(np.isin(label, [label[order[0]], label[full[np.sum(label == label[order[0]])]]])))
    assert order[:k].tolist() == full[:k].tolist()
    placed = set(order[:k].tolist())
    assert order[k:].tolist() == [int(v) for v in by_deg if int(v) not in placed]
