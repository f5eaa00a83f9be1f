"""Pins for the oracle's aggregate-max and its adjoint."""
import numpy as np

import oracle
from ag_inputs import from_edges, planted_partition, directed_random, features
from helpers import dense_from_csr


def test_max_against_dense_brute_force_directed():
    g = directed_random(60, 3.0, 4, weighted=False, self_loops=False)     # has empty rows
    H = features(g.n, 5, 1)
    Y, arg = oracle.spmax(g.rowptr, g.colidx, H)
    A = dense_from_csr(g.rowptr, g.colidx, None) != 0
    assert (~A.any(axis=1)).any()                                          # the empty-row case is present
    for i in range(g.n):
        for k in range(5):
            js = np.nonzero(A[i])[0]
            if js.size == 0:
                assert Y[i, k] == 0.0 and arg[i, k] == -1
            else:
                assert Y[i, k] == H[js, k].max()
                assert arg[i, k] == js[np.argmax(H[js, k])]                # argmax returns the first = smallest j


def test_max_star_closed_form_and_ties():
    # star with self loops: leaves see {centre, self}, the centre sees everyone
    n = 7
    g = from_edges(n, np.zeros(n - 1, int), np.arange(1, n))
    H = np.arange(n, dtype=np.float32)[:, None] * np.array([[1.0, -1.0]], np.float32)
    Y, arg = oracle.spmax(g.rowptr, g.colidx, H)
    assert Y[:, 0].tolist() == [6.0] + [float(i) for i in range(1, n)]     # column 0 grows with the id
    assert arg[:, 0].tolist() == [6] + list(range(1, n))
    assert Y[:, 1].tolist() == [0.0] * n                                   # column 1 falls: the centre (0) wins
    assert arg[:, 1].tolist() == [0] * n
    Hc = np.ones((n, 1), np.float32)                                       # all equal: smallest source wins
    Y, arg = oracle.spmax(g.rowptr, g.colidx, Hc)
    assert arg[:, 0].tolist() == [0] * n and np.all(Y == 1.0)


def test_max_adjoint_is_the_gradient_by_central_differences():
    g = directed_random(25, 3.0, 9, weighted=False)
    H = features(g.n, 3, 2).astype(np.float64)
    G = features(g.n, 3, 3)
    _, arg = oracle.spmax(g.rowptr, g.colidx, H.astype(np.float32))
    D, S = oracle.spmax_t(arg, G)

    def f(Hx):                                       # scalar whose gradient w.r.t. H is the adjoint applied to G
        A = dense_from_csr(g.rowptr, g.colidx, None) != 0
        tot = 0.0
        for i in range(g.n):
            js = np.nonzero(A[i])[0]
            if js.size:
                tot += float((G[i] * Hx[js].max(axis=0)).sum())
        return tot
    H32 = H.astype(np.float32).astype(np.float64)
    eps = 1e-4                                       # far below the gaps between random values
    num = np.zeros_like(H32)
    for j in range(g.n):
        for k in range(3):
            Hp, Hm = H32.copy(), H32.copy()
            Hp[j, k] += eps
            Hm[j, k] -= eps
            num[j, k] = (f(Hp) - f(Hm)) / (2 * eps)
    np.testing.assert_allclose(D, num, rtol=1e-6, atol=1e-7)
    assert np.all(S >= np.abs(D) - 1e-12)


def test_max_adjoint_conserves_mass():
    g = planted_partition(4, 32, 6, 0.7, 5)
    H, G = features(g.n, 8, 1), features(g.n, 8, 2)
    _, arg = oracle.spmax(g.rowptr, g.colidx, H)
    D, _ = oracle.spmax_t(arg, G)
    np.testing.assert_allclose(D.sum(axis=0), G.astype(np.float64).sum(axis=0), rtol=1e-12, atol=1e-12)
