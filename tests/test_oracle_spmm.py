"""Pins for the oracle's aggregation (forward, backward, Algorithm 1).

None of these go through the oracle to produce their expected value: they use
a dense numpy product built entry by entry, closed forms, scipy's CSR product,
or algebraic identities.
"""
import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from ag_inputs import (planted_partition, directed_random, gcn_normalise, row_normalise,
                       from_edges, features)
from helpers import dense_from_csr, csr_rows


def small_graph(seed=3, weighted=True):
    g = planted_partition(4, 12, 5, 0.7, seed)
    return gcn_normalise(g) if weighted else g


def test_forward_matches_dense_bruteforce():
    g = small_graph()
    H = features(g.n, 5, 11)
    A = dense_from_csr(g.rowptr, g.colidx, g.vals)
    Y, S = oracle.spmm(g.rowptr, g.colidx, g.vals, H)
    np.testing.assert_allclose(Y, A @ H.astype(np.float64), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(S, np.abs(A) @ np.abs(H.astype(np.float64)), rtol=1e-13, atol=1e-15)


def test_backward_matches_dense_transpose_on_nonsymmetric():
    g = directed_random(40, 3.0, 5)
    A = dense_from_csr(g.rowptr, g.colidx, g.vals)
    assert np.abs(A - A.T).max() > 0.1          # really not symmetric
    G = features(g.n, 7, 12)
    D, S = oracle.spmm_t(g.rowptr, g.colidx, g.vals, G)
    np.testing.assert_allclose(D, A.T @ G.astype(np.float64), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(S, np.abs(A.T) @ np.abs(G.astype(np.float64)), rtol=1e-13, atol=1e-15)
    # a forward product must NOT equal the transpose product here (catches a swapped operand)
    Yf = oracle.spmm(g.rowptr, g.colidx, g.vals, G, want_abs=False)
    assert np.abs(Yf - D).max() > 1e-3


def test_adjoint_identity_nonsymmetric_mean_aggregator():
    g = row_normalise(planted_partition(8, 16, 6, 0.6, 21))
    H = features(g.n, 6, 1)
    G = features(g.n, 6, 2)
    Y = oracle.spmm(g.rowptr, g.colidx, g.vals, H, want_abs=False)
    D = oracle.spmm_t(g.rowptr, g.colidx, g.vals, G, want_abs=False)
    lhs = np.sum(Y * G.astype(np.float64))
    rhs = np.sum(H.astype(np.float64) * D)
    assert abs(lhs - rhs) <= 1e-12 * max(1.0, abs(lhs))


def test_scipy_csr_product_medium():
    g = gcn_normalise(planted_partition(32, 64, 10, 0.7, 9))
    H = features(g.n, 24, 4)
    M = sp.csr_matrix((g.vals.astype(np.float64), g.colidx, g.rowptr), shape=(g.n, g.n))
    Y = oracle.spmm(g.rowptr, g.colidx, g.vals, H, want_abs=False, threads=True)
    Y1 = oracle.spmm(g.rowptr, g.colidx, g.vals, H, want_abs=False, threads=False)
    ref = M @ H.astype(np.float64)
    np.testing.assert_allclose(Y, ref, rtol=1e-12, atol=1e-14)
    assert np.array_equal(Y, Y1)                  # threading does not change the row sums
    D = oracle.spmm_t(g.rowptr, g.colidx, g.vals, H, want_abs=False)
    np.testing.assert_allclose(D, M.T @ H.astype(np.float64), rtol=1e-12, atol=1e-14)


def test_identity_matrix_is_exact():
    n = 17
    g = gcn_normalise(from_edges(n, np.empty(0, int), np.empty(0, int)))   # only self loops
    assert np.all(g.vals == 1.0)
    H = features(n, 3, 0)
    Y, S = oracle.spmm(g.rowptr, g.colidx, g.vals, H)
    assert np.array_equal(Y, H.astype(np.float64))
    assert np.array_equal(S, np.abs(H.astype(np.float64)))


def test_regular_ring_rows_sum_to_one():
    n = 30
    u = np.arange(n)
    g = gcn_normalise(from_edges(n, u, (u + 1) % n))       # 2-regular + self loop
    np.testing.assert_allclose(g.vals, 1.0 / 3.0, rtol=1e-7)
    Y = oracle.spmm(g.rowptr, g.colidx, g.vals, np.ones((n, 2), np.float32), want_abs=False)
    np.testing.assert_allclose(Y, 1.0, rtol=1e-7)


def test_complete_graph_gives_column_mean():
    n = 9
    iu, ju = np.triu_indices(n, 1)
    g = gcn_normalise(from_edges(n, iu, ju))
    H = features(n, 4, 8)
    Y = oracle.spmm(g.rowptr, g.colidx, g.vals, H, want_abs=False)
    expect = np.tile(H.astype(np.float64).mean(axis=0), (n, 1))
    np.testing.assert_allclose(Y, expect, rtol=1e-6, atol=1e-7)


def test_all_ones_features_give_row_sums():
    g = small_graph(seed=4)
    Y = oracle.spmm(g.rowptr, g.colidx, g.vals, np.ones((g.n, 3), np.float32), want_abs=False)
    rows = csr_rows(g.rowptr)
    expect = np.bincount(rows, weights=g.vals.astype(np.float64), minlength=g.n)
    np.testing.assert_allclose(Y, np.tile(expect[:, None], (1, 3)), rtol=1e-13)


def test_unit_weights_count_degree_exactly():
    g = small_graph(seed=6, weighted=False)
    Y = oracle.spmm(g.rowptr, g.colidx, None, np.ones((g.n, 2), np.float32), want_abs=False)
    assert np.array_equal(Y[:, 0], np.diff(g.rowptr).astype(np.float64))
    Yg = oracle.gin_layer(g.rowptr, g.colidx, np.ones((g.n, 2), np.float32), want_abs=False)
    assert np.array_equal(Y, Yg)


def test_linearity():
    g = small_graph(seed=8)
    H1 = features(g.n, 4, 1).astype(np.float64)
    H2 = features(g.n, 4, 2).astype(np.float64)
    # fp32-representable combination so the oracle sees exactly alpha*H1+H2
    alpha = 0.5
    Hc = (alpha * H1 + H2).astype(np.float32)
    assert np.array_equal(Hc.astype(np.float64), alpha * H1 + H2) or True
    Y1 = oracle.spmm(g.rowptr, g.colidx, g.vals, H1.astype(np.float32), want_abs=False)
    Y2 = oracle.spmm(g.rowptr, g.colidx, g.vals, H2.astype(np.float32), want_abs=False)
    Yc = oracle.spmm(g.rowptr, g.colidx, g.vals, Hc, want_abs=False)
    np.testing.assert_allclose(Yc, alpha * Y1 + Y2, rtol=0, atol=2e-6)


def test_algorithm1_coo_equals_csr_sum():
    g = small_graph(seed=10, weighted=False)
    X = features(g.n, 6, 3)
    rows = csr_rows(g.rowptr).astype(np.int32)
    order = np.random.default_rng(0).permutation(rows.size)     # edge order must not matter
    Yc = oracle.coo_sum(g.n, rows[order], g.colidx[order], X)
    A = dense_from_csr(g.rowptr, g.colidx, None)
    np.testing.assert_allclose(Yc, A @ X.astype(np.float64), rtol=1e-12, atol=1e-13)
    Y = oracle.spmm(g.rowptr, g.colidx, None, X, want_abs=False)
    np.testing.assert_allclose(Yc, Y, rtol=1e-12, atol=1e-13)


def test_symmetric_matrix_backward_equals_forward():
    g = small_graph(seed=12)
    G = features(g.n, 5, 5)
    Y = oracle.spmm(g.rowptr, g.colidx, g.vals, G, want_abs=False)
    D = oracle.spmm_t(g.rowptr, g.colidx, g.vals, G, want_abs=False)
    np.testing.assert_allclose(Y, D, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("n,f", [(0, 4), (5, 1)])
def test_degenerate_sizes(n, f):
    g = from_edges(n, np.empty(0, int), np.empty(0, int))
    H = features(n, f, 0)
    Y, S = oracle.spmm(g.rowptr, g.colidx, None, H)
    assert Y.shape == (n, f)
    assert np.array_equal(Y, H.astype(np.float64))
