"""Pins for the oracle's GCN training step and GIN layer."""
import math

import numpy as np

import oracle
from ag_inputs import planted_partition, gcn_normalise, row_normalise, features, glorot_uniform, labels
from helpers import dense_from_csr


def setup(n_comm=2, size=16, fin=6, hid=5, ncls=4, seed=3, norm=gcn_normalise):
    g = norm(planted_partition(n_comm, size, 4, 0.7, seed))
    X = features(g.n, fin, 1)
    W1 = glorot_uniform(fin, hid, 2)
    W2 = glorot_uniform(hid, ncls, 3)
    b1 = (0.1 * features(1, hid, 4)[0]).astype(np.float32)
    b2 = (0.1 * features(1, ncls, 5)[0]).astype(np.float32)
    y = labels(g.n, ncls, 6)
    return g, X, W1, b1, W2, b2, y


def test_zero_weights_loss_is_log_classes():
    g, X, W1, b1, W2, b2, y = setup(ncls=16)
    r = oracle.gcn_step(g.rowptr, g.colidx, g.vals, X, W1 * 0, b1 * 0, W2 * 0, b2 * 0, y)
    assert abs(r.loss - math.log(16.0)) < 1e-14
    assert abs(r.loss - 2.772588722239781) < 1e-14


def test_forward_against_dense_formula():
    g, X, W1, b1, W2, b2, y = setup()
    A = dense_from_csr(g.rowptr, g.colidx, g.vals)
    r = oracle.gcn_step(g.rowptr, g.colidx, g.vals, X, W1, b1, W2, b2, y)
    f = np.float64
    Z = A @ (np.maximum(A @ X.astype(f) @ W1.astype(f) + b1.astype(f), 0) @ W2.astype(f)) + b2.astype(f)
    np.testing.assert_allclose(r.Z, Z, rtol=1e-12, atol=1e-14)
    p = np.exp(Z) / np.exp(Z).sum(1, keepdims=True)
    loss = -np.mean(np.log(p[np.arange(g.n), y]))
    assert abs(loss - r.loss) < 1e-12


def _loss(g, X, W1, b1, W2, b2, y):
    return oracle.gcn_step(g.rowptr, g.colidx, g.vals, X, W1, b1, W2, b2, y).loss


def test_gradients_by_central_differences_nonsymmetric_A():
    # a non-symmetric (row-normalised) adjacency makes a forgotten transpose visible
    g, X, W1, b1, W2, b2, y = setup(norm=row_normalise)
    f = np.float64
    W1, b1, W2, b2 = (a.astype(f) for a in (W1, b1, W2, b2))
    r = oracle.gcn_step(g.rowptr, g.colidx, g.vals, X, W1, b1, W2, b2, y)
    eps = 1e-6
    for name, arr, grad in (("W1", W1, r.dW1), ("b1", b1, r.db1), ("W2", W2, r.dW2), ("b2", b2, r.db2)):
        num = np.zeros_like(arr)
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = arr[idx]
            arr[idx] = old + eps
            lp = _loss(g, X, W1, b1, W2, b2, y)
            arr[idx] = old - eps
            lm = _loss(g, X, W1, b1, W2, b2, y)
            arr[idx] = old
            num[idx] = (lp - lm) / (2 * eps)
        np.testing.assert_allclose(grad, num, rtol=2e-5, atol=2e-9, err_msg=name)


def test_gin_layer_is_A_plus_I_sum():
    g = planted_partition(3, 10, 4, 0.6, 9)
    H = features(g.n, 3, 2)
    A = dense_from_csr(g.rowptr, g.colidx, None)
    assert np.all(np.diag(A) == 1.0)
    Y, S = oracle.gin_layer(g.rowptr, g.colidx, H)
    np.testing.assert_allclose(Y, A @ H.astype(np.float64), rtol=1e-13, atol=1e-15)


# --------------------------------------------------------------------------- #
# GIN training step
# --------------------------------------------------------------------------- #
def gin_setup(widths, seed=5, directed=False):
    from ag_inputs import directed_random
    g = directed_random(40, 3.0, seed, weighted=False) if directed else planted_partition(2, 16, 4, 0.7, seed)
    X = features(g.n, widths[0], 1)
    Ws = [glorot_uniform(widths[l], widths[l + 1], 10 + l) for l in range(len(widths) - 1)]
    bs = [(0.1 * features(1, widths[l + 1], 20 + l)[0]).astype(np.float32) for l in range(len(widths) - 1)]
    y = labels(g.n, widths[-1], 6)
    return g, X, Ws, bs, y


def test_gin_one_layer_is_softmax_regression_on_aggregated_features():
    # L = 1: logits = ((A + eps I) X) W + b; the gradient of softmax regression has the closed
    # form  dW = M^T (softmax - onehot) / n  with M the aggregated features
    g, X, Ws, bs, y = gin_setup([5, 4])
    eps = 0.25
    r = oracle.gin_step(g.rowptr, g.colidx, None, X, Ws, bs, y, eps=eps)
    A = dense_from_csr(g.rowptr, g.colidx, None)
    M = (A + eps * np.eye(g.n)) @ X.astype(np.float64)
    Z = M @ Ws[0].astype(np.float64) + bs[0].astype(np.float64)
    np.testing.assert_allclose(r.Z, Z, rtol=1e-12, atol=1e-14)
    p = np.exp(Z) / np.exp(Z).sum(1, keepdims=True)
    onehot = np.eye(4)[y]
    np.testing.assert_allclose(r.dW[0], M.T @ (p - onehot) / g.n, rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(r.db[0], (p - onehot).sum(0) / g.n, rtol=1e-11, atol=1e-14)
    assert abs(r.loss + np.mean(np.log(p[np.arange(g.n), y]))) < 1e-12


def test_gin_forward_against_dense_formula_three_layers():
    g, X, Ws, bs, y = gin_setup([6, 5, 7, 3])
    A = dense_from_csr(g.rowptr, g.colidx, None)
    f = np.float64
    H = X.astype(f)
    for l in range(3):
        H = A @ H @ Ws[l].astype(f) + bs[l].astype(f)
        if l < 2:
            H = np.maximum(H, 0)
    r = oracle.gin_step(g.rowptr, g.colidx, None, X, Ws, bs, y)
    np.testing.assert_allclose(r.Z, H, rtol=1e-12, atol=1e-14)


def test_gin_zero_weights_loss_is_log_classes():
    g, X, Ws, bs, y = gin_setup([6, 5, 8])
    r = oracle.gin_step(g.rowptr, g.colidx, None, X, [w * 0 for w in Ws], [b * 0 for b in bs], y)
    assert abs(r.loss - math.log(8.0)) < 1e-14


def test_gin_gradients_by_central_differences_directed_graph():
    # a directed (non-symmetric) pattern makes a forgotten transpose visible; eps != 0 covers the self term
    g, X, Ws, bs, y = gin_setup([4, 5, 3, 3], directed=True)
    f = np.float64
    Ws = [w.astype(f) for w in Ws]
    bs = [b.astype(f) for b in bs]
    eps = 0.5
    r = oracle.gin_step(g.rowptr, g.colidx, None, X, Ws, bs, y, eps=eps)
    h = 1e-6
    for l in range(3):
        for name, arr, grad in (("W", Ws[l], r.dW[l]), ("b", bs[l], r.db[l])):
            num = np.zeros_like(arr)
            it = np.nditer(arr, flags=["multi_index"])
            for _ in it:
                idx = it.multi_index
                old = arr[idx]
                arr[idx] = old + h
                lp = oracle.gin_step(g.rowptr, g.colidx, None, X, Ws, bs, y, eps=eps).loss
                arr[idx] = old - h
                lm = oracle.gin_step(g.rowptr, g.colidx, None, X, Ws, bs, y, eps=eps).loss
                arr[idx] = old
                num[idx] = (lp - lm) / (2 * h)
            np.testing.assert_allclose(grad, num, rtol=2e-5, atol=2e-9, err_msg=f"{name}{l}")
