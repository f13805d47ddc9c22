"""Pins for the oracle's normalised-CSR builder and its sparse aggregation.

Nothing here re-types the oracle's own loops: the checks are dense brute force from the
definition A^ = D~^-1/2 (A + I) D~^-1/2 on tiny graphs, graphs whose A^ has a closed form,
invariants that hold for every graph, and a library routine (scipy) as a special case.
"""
import numpy as np
import pytest
import scipy.sparse as sp

import oracle

RNG = np.random.default_rng(20240811)


def messy_edges(n, m, rng):
    """Directed pairs with repeats, both orientations and self pairs mixed in."""
    src = rng.integers(0, n, size=m)
    dst = rng.integers(0, n, size=m)
    rep = rng.integers(0, m, size=m // 3)
    src = np.concatenate([src, src[rep], dst[rep][: m // 6]])
    dst = np.concatenate([dst, dst[rep], src[rep][: m // 6]])
    return src.astype(np.int64), dst.astype(np.int64)


def dense_normalised(src, dst, n, symmetrize=True, loops=True):
    """A^ straight from the definition, as a dense matrix."""
    A = np.zeros((n, n))
    for u, v in zip(src, dst):
        if u != v:
            A[u, v] = 1.0
            if symmetrize:
                A[v, u] = 1.0
    if loops:
        A += np.eye(n)
    d = A.sum(axis=1)
    d[d == 0] = 1.0
    return A, (A / np.sqrt(d)[:, None]) / np.sqrt(d)[None, :]


def to_dense(g):
    M = np.zeros((g.n, g.n))
    for v in range(g.n):
        for e in range(g.rowptr[v], g.rowptr[v + 1]):
            assert M[v, g.colidx[e]] == 0.0, "duplicate stored entry"
            M[v, g.colidx[e]] = g.vals[e]
    return M


@pytest.mark.parametrize("n,m", [(1, 0), (2, 1), (5, 7), (17, 40), (33, 200), (64, 300), (64, 2000)])
@pytest.mark.parametrize("flags", [3, 2, 1, 0])
def test_dense_brute_force(n, m, flags):
    rng = np.random.default_rng(n * 1000 + m + flags)
    src, dst = messy_edges(n, m, rng) if m else (np.zeros(0, np.int64), np.zeros(0, np.int64))
    g = oracle.build_norm_csr(src, dst, n, flags)
    A, Ahat = dense_normalised(src, dst, n, symmetrize=bool(flags & 1), loops=bool(flags & 2))
    M = to_dense(g)
    assert np.array_equal(M != 0, A != 0)
    np.testing.assert_allclose(M, Ahat, rtol=1e-15, atol=0)
    assert np.array_equal(g.deg, (A != 0).sum(axis=1))
    X = rng.standard_normal((n, 5))
    np.testing.assert_allclose(oracle.spmm(g, X), Ahat @ X, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(oracle.spmm(g, X, transpose=True), Ahat.T @ X, rtol=1e-13, atol=1e-14)
    rows = rng.integers(0, n, size=7)
    np.testing.assert_allclose(oracle.spmm_rows(g, X, rows), (Ahat @ X)[rows], rtol=1e-13, atol=1e-14)


def test_structure_invariants():
    n, m = 500, 3000
    src, dst = messy_edges(n, m, RNG)
    g = oracle.build_norm_csr(src, dst, n)
    und = {(min(u, v), max(u, v)) for u, v in zip(src, dst) if u != v}
    assert g.rowptr[0] == 0 and np.all(np.diff(g.rowptr) >= 1)
    assert g.nnz == 2 * len(und) + n == g.deg.sum()
    assert np.array_equal(g.deg, np.diff(g.rowptr))
    pairs = set()
    for v in range(n):
        cols = g.colidx[g.rowptr[v]:g.rowptr[v + 1]]
        assert np.all(np.diff(cols) > 0)            # strictly ascending: sorted and distinct
        assert v in cols                            # exactly one diagonal (distinctness gives "one")
        pairs |= {(v, int(c)) for c in cols}
    assert all((c, v) in pairs for v, c in pairs)   # symmetric pattern
    # symmetric values, bit for bit
    M = sp.csr_matrix((g.vals, g.colidx, g.rowptr), shape=(n, n))
    assert (M != M.T).nnz == 0
    np.testing.assert_array_equal(g.dinv, 1.0 / np.sqrt(g.deg.astype(np.float64)))


@pytest.mark.parametrize("flags", [3, 2])
def test_fixed_point_invariant(flags):
    """A^ (D~^1/2 1) = D~^1/2 1 for any pattern whose D~ is its row sum."""
    n = 300
    src, dst = messy_edges(n, 2500, RNG)
    g = oracle.build_norm_csr(src, dst, n, flags)
    s = np.sqrt(g.deg.astype(np.float64))[:, None]
    np.testing.assert_allclose(oracle.spmm(g, s), s, rtol=1e-13)


def test_empty_graph_is_identity():
    n = 9
    g = oracle.build_norm_csr(np.zeros(0, np.int64), np.zeros(0, np.int64), n)
    X = RNG.standard_normal((n, 4))
    np.testing.assert_array_equal(oracle.spmm(g, X), X)
    assert np.array_equal(g.colidx, np.arange(n)) and np.all(g.vals == 1.0)


def test_complete_graph_is_mean():
    n = 12
    iu = np.triu_indices(n, 1)
    g = oracle.build_norm_csr(iu[0], iu[1], n)
    X = RNG.standard_normal((n, 3))
    np.testing.assert_allclose(oracle.spmm(g, X), np.tile(X.mean(axis=0), (n, 1)), rtol=1e-13)


def test_ring_is_three_tap_mean():
    n = 11
    v = np.arange(n)
    g = oracle.build_norm_csr(v, (v + 1) % n, n)
    X = RNG.standard_normal((n, 3))
    want = (np.roll(X, 1, axis=0) + X + np.roll(X, -1, axis=0)) / 3.0
    np.testing.assert_allclose(oracle.spmm(g, X), want, rtol=1e-13)


def test_star_closed_form():
    n = 10  # node 0 is the centre
    g = oracle.build_norm_csr(np.zeros(n - 1, np.int64), np.arange(1, n), n)
    X = RNG.standard_normal((n, 2))
    Z = oracle.spmm(g, X)
    centre = X[0] / n + X[1:].sum(axis=0) / np.sqrt(2.0 * n)
    np.testing.assert_allclose(Z[0], centre, rtol=1e-13)
    for leaf in range(1, n):
        np.testing.assert_allclose(Z[leaf], X[leaf] / 2.0 + X[0] / np.sqrt(2.0 * n), rtol=1e-13)


def test_regular_graph():
    # 4-regular circulant: A^ = (A + I) / 5
    n = 15
    v = np.arange(n)
    src = np.concatenate([v, v]); dst = np.concatenate([(v + 1) % n, (v + 2) % n])
    g = oracle.build_norm_csr(src, dst, n)
    assert np.all(g.deg == 5)
    np.testing.assert_allclose(g.vals, 0.2, rtol=1e-15)


def test_spectral_radius_is_one():
    n = 40
    src, dst = messy_edges(n, 120, RNG)
    g = oracle.build_norm_csr(src, dst, n)
    eig = np.linalg.eigvalsh(to_dense(g))
    assert abs(eig.max() - 1.0) < 1e-12 and eig.min() > -1.0 - 1e-12


def test_concat_of_slice_aggregations_is_unsliced_aggregation():
    n, F = 200, 37
    src, dst = messy_edges(n, 900, RNG)
    g = oracle.build_norm_csr(src, dst, n)
    X = RNG.standard_normal((n, F))
    full = oracle.spmm(g, X)
    for p in (2, 3, 5):
        sl, c = oracle.slice_strategy(F, p)
        for s, e in sl:                       # column for column, bit for bit (same sums, same order)
            np.testing.assert_array_equal(oracle.spmm(g, X[:, s:e]), full[:, s:e])


def test_linearity_and_adjoint_on_directed_graph():
    n = 150
    src, dst = messy_edges(n, 700, RNG)
    g = oracle.build_norm_csr(src, dst, n, oracle.ADD_SELF_LOOPS)   # not symmetrised: A^ != A^^T
    X, Y, G = (RNG.standard_normal((n, 6)) for _ in range(3))
    a, b = 0.37, -1.9
    np.testing.assert_allclose(oracle.spmm(g, a * X + b * Y), a * oracle.spmm(g, X) + b * oracle.spmm(g, Y), rtol=1e-12, atol=1e-13)
    lhs = np.sum(oracle.spmm(g, X) * G)
    rhs = np.sum(X * oracle.spmm(g, G, transpose=True))
    assert abs(lhs - rhs) <= 1e-12 * abs(lhs)
    assert not np.allclose(oracle.spmm(g, X), oracle.spmm(g, X, transpose=True))


def test_scipy_cross_check():
    n = 3000
    src, dst = messy_edges(n, 30000, RNG)
    g = oracle.build_norm_csr(src, dst, n)
    # pattern built independently with scipy from the raw pairs
    keep = src != dst
    A = sp.coo_matrix((np.ones(keep.sum()), (src[keep], dst[keep])), shape=(n, n)).tocsr()
    A = ((A + A.T + sp.identity(n)) > 0).astype(np.float64).tocsr()
    A.sort_indices()
    assert np.array_equal(A.indptr, g.rowptr) and np.array_equal(A.indices, g.colidx)
    d = np.asarray(A.sum(axis=1)).ravel()
    Ahat = sp.diags(d ** -0.5) @ A @ sp.diags(d ** -0.5)
    X = RNG.standard_normal((n, 8))
    np.testing.assert_allclose(oracle.spmm(g, X), Ahat @ X, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(oracle.spmm(g, X, transpose=True), Ahat.T @ X, rtol=1e-12, atol=1e-13)


def test_rejects_bad_input():
    with pytest.raises(ValueError):
        oracle.build_norm_csr([0, 5], [1, 2], 4)          # node id out of range
    with pytest.raises(ValueError):
        oracle.build_norm_csr([0, -1], [1, 2], 4)
    with pytest.raises(ValueError):
        oracle.build_norm_csr([0], [1], 4, flags=8)       # unknown flag
    with pytest.raises(ValueError):
        oracle.build_norm_csr([], [], 0)
