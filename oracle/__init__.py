"""CPU oracle (fp64) for the AdaptGear aggregation path.  TEST INFRASTRUCTURE ONLY.

Only `tests/`, `__graft_entry__.smoke()` and the `cpu_baseline` leg of
`bench.py` may import this package.  It never imports the HIP package and the
HIP package never imports it.

The heavy loops live in `ag_oracle.c` (plain C, compiled with gcc into
`libag_oracle.so` next to this file); this module marshals numpy arrays into
it and adds the dense-layer arithmetic of the GCN / GIN steps in numpy fp64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from types import SimpleNamespace

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libag_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile ag_oracle.c with gcc (OpenMP on) into libag_oracle.so."""
    src = os.path.join(_HERE, "ag_oracle.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-Wall", "-o", _LIB_PATH, src, "-lm"])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB_PATH)
        _lib.orc_num_threads.restype = ctypes.c_int
        _lib.orc_reorder.restype = ctypes.c_int
        _lib.orc_reorder_method.restype = ctypes.c_int
        _lib.orc_split.restype = ctypes.c_int
    return _lib


def _p(a, ct):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ct))


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def num_threads() -> int:
    return int(_load().orc_num_threads())


def spmm(rowptr, colidx, vals, H, *, want_abs=True, threads=True):
    """Y = A.H in fp64 from fp32 inputs; also S = sum |a_ij h_jk| when asked.

    Aggregate-sum over each destination row's source neighbours (paper Sec. 2.1).
    """
    lib = _load()
    rowptr, colidx, vals, H = _i32(rowptr), _i32(colidx), _f32(vals), _f32(H)
    n, F = rowptr.size - 1, H.shape[1]
    Y = np.empty((n, F), dtype=np.float64)
    S = np.empty((n, F), dtype=np.float64) if want_abs else None
    lib.orc_spmm(ctypes.c_int64(n), _p(rowptr, ctypes.c_int32), _p(colidx, ctypes.c_int32),
                 _p(vals, ctypes.c_float), ctypes.c_int32(F), _p(H, ctypes.c_float),
                 _p(Y, ctypes.c_double), _p(S, ctypes.c_double), ctypes.c_int32(1 if threads else 0))
    return (Y, S) if want_abs else Y


def spmm_t(rowptr, colidx, vals, G, *, want_abs=True, threads=True):
    """dH = A^T.G in fp64 (the backward of spmm)."""
    lib = _load()
    rowptr, colidx, vals, G = _i32(rowptr), _i32(colidx), _f32(vals), _f32(G)
    n, F = rowptr.size - 1, G.shape[1]
    D = np.empty((n, F), dtype=np.float64)
    S = np.empty((n, F), dtype=np.float64) if want_abs else None
    lib.orc_spmm_t(ctypes.c_int64(n), _p(rowptr, ctypes.c_int32), _p(colidx, ctypes.c_int32),
                   _p(vals, ctypes.c_float), ctypes.c_int32(F), _p(G, ctypes.c_float),
                   _p(D, ctypes.c_double), _p(S, ctypes.c_double), ctypes.c_int32(1 if threads else 0))
    return (D, S) if want_abs else D


def coo_sum(n, row, col, X):
    """Algorithm 1 of the paper, run serially: Y[dst] += X[src] for every edge."""
    lib = _load()
    row, col, X = _i32(row), _i32(col), _f32(X)
    F = X.shape[1]
    Y = np.empty((n, F), dtype=np.float64)
    lib.orc_coo_sum(ctypes.c_int64(n), ctypes.c_int64(row.size), _p(row, ctypes.c_int32),
                    _p(col, ctypes.c_int32), ctypes.c_int32(F), _p(X, ctypes.c_float),
                    _p(Y, ctypes.c_double))
    return Y


def spmax(rowptr, colidx, H):
    """Aggregate-max (paper Sec. 2.1): Y[i][k] = max over row i's stored sources of H[j][k] and
    the smallest source attaining it; empty rows give 0 / -1.  Edge values play no part."""
    lib = _load()
    rowptr, colidx, H = _i32(rowptr), _i32(colidx), _f32(H)
    n, F = rowptr.size - 1, H.shape[1]
    Y = np.empty((n, F), dtype=np.float64)
    arg = np.empty((n, F), dtype=np.int32)
    lib.orc_spmax(ctypes.c_int64(n), _p(rowptr, ctypes.c_int32), _p(colidx, ctypes.c_int32),
                  ctypes.c_int32(F), _p(H, ctypes.c_float), _p(Y, ctypes.c_double), _p(arg, ctypes.c_int32))
    return Y, arg


def spmax_t(arg, G):
    """Adjoint of spmax: dH[j][k] = sum of G[i][k] over the rows i whose maximum came from j;
    also the same sum of |G| for the tolerance."""
    lib = _load()
    arg, G = _i32(arg), _f32(G)
    n, F = G.shape
    D = np.empty((n, F), dtype=np.float64)
    S = np.empty((n, F), dtype=np.float64)
    lib.orc_spmax_t(ctypes.c_int64(n), ctypes.c_int32(F), _p(arg, ctypes.c_int32), _p(G, ctypes.c_float),
                    _p(D, ctypes.c_double), _p(S, ctypes.c_double))
    return D, S


def reorder(rowptr, colidx, *, block_cap=128, min_block=16, sweeps=8, max_levels=12, order_levels=3, method=0):
    """Community reordering (paper Sec. 2.2 / 4.2); see orc_reorder_method in ag_oracle.c.
    method 0 = multilevel label propagation, 1 = agglomeration by integer modularity gain."""
    lib = _load()
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    n = rowptr.size - 1
    perm = np.empty(n, np.int32)
    iperm = np.empty(n, np.int32)
    blk = np.empty(n + 1, np.int32)
    comm = np.empty(n, np.int32)
    nb = ctypes.c_int32(0)
    rc = lib.orc_reorder_method(ctypes.c_int64(n), _p(rowptr, ctypes.c_int32), _p(colidx, ctypes.c_int32),
                         ctypes.c_int32(method), ctypes.c_int32(block_cap), ctypes.c_int32(min_block), ctypes.c_int32(sweeps),
                         ctypes.c_int32(max_levels), ctypes.c_int32(order_levels),
                         _p(perm, ctypes.c_int32), _p(iperm, ctypes.c_int32),
                         _p(blk, ctypes.c_int32), ctypes.byref(nb), _p(comm, ctypes.c_int32))
    if rc:
        raise MemoryError("orc_reorder failed")
    return SimpleNamespace(perm=perm, iperm=iperm, blk_ptr=blk[: nb.value + 1].copy(), comm=comm)


def split(rowptr, colidx, vals, perm, iperm, blk_ptr):
    """Decompose the reordered matrix into intra / inter CSR parts (paper Sec. 3.3)."""
    lib = _load()
    rowptr, colidx, vals = _i32(rowptr), _i32(colidx), _f32(vals)
    perm, iperm, blk_ptr = _i32(perm), _i32(iperm), _i32(blk_ptr)
    n, nnz = rowptr.size - 1, int(rowptr[-1])
    irp, orp = np.empty(n + 1, np.int32), np.empty(n + 1, np.int32)
    ic, oc = np.empty(nnz, np.int32), np.empty(nnz, np.int32)
    iv, ov = np.empty(nnz, np.float32), np.empty(nnz, np.float32)
    rc = lib.orc_split(ctypes.c_int64(n), _p(rowptr, ctypes.c_int32), _p(colidx, ctypes.c_int32),
                       _p(vals, ctypes.c_float), _p(perm, ctypes.c_int32), _p(iperm, ctypes.c_int32),
                       _p(blk_ptr, ctypes.c_int32), ctypes.c_int32(blk_ptr.size - 1),
                       _p(irp, ctypes.c_int32), _p(ic, ctypes.c_int32), _p(iv, ctypes.c_float),
                       _p(orp, ctypes.c_int32), _p(oc, ctypes.c_int32), _p(ov, ctypes.c_float))
    if rc:
        raise MemoryError("orc_split failed")
    ni, no = int(irp[-1]), int(orp[-1])
    return SimpleNamespace(intra_rowptr=irp, intra_col=ic[:ni].copy(), intra_val=iv[:ni].copy(),
                           inter_rowptr=orp, inter_col=oc[:no].copy(), inter_val=ov[:no].copy())


# --------------------------------------------------------------------------- #
# model steps (numpy fp64 around the C aggregation)
# --------------------------------------------------------------------------- #
def gin_layer(rowptr, colidx, H, *, want_abs=True):
    """GIN sum aggregation with eps = 0: (A + I).H where the stored pattern
    already carries the unit diagonal (paper Sec. 2.1 aggregate-sum; Sec. 5)."""
    return spmm(rowptr, colidx, None, H, want_abs=want_abs)


def gcn_step(rowptr, colidx, vals, X, W1, b1, W2, b2, labels):
    """Two-layer GCN forward + backward in fp64 (paper Sec. 5 "Benchmarks").

    Layer 1 aggregates first (P = A.X, H1 = relu(P W1 + b1)); layer 2 transforms
    first (Q = H1 W2, Z = A.Q + b2); loss = mean softmax cross-entropy.  Returns
    every intermediate and every gradient.
    """
    f = np.float64
    X32 = np.asarray(X, np.float32)
    W1, b1, W2, b2 = (np.asarray(a, f) for a in (W1, b1, W2, b2))
    n = X32.shape[0]
    P = spmm(rowptr, colidx, vals, X32, want_abs=False)
    pre1 = P @ W1 + b1
    H1 = np.maximum(pre1, 0.0)
    Q = H1 @ W2
    Z = _spmm64(rowptr, colidx, vals, Q) + b2
    zmax = Z.max(axis=1, keepdims=True)
    ez = np.exp(Z - zmax)
    sm = ez / ez.sum(axis=1, keepdims=True)
    lse = np.log(ez.sum(axis=1)) + zmax[:, 0]
    loss = float(np.mean(lse - Z[np.arange(n), labels]))
    dZ = sm.copy()
    dZ[np.arange(n), labels] -= 1.0
    dZ /= n
    db2 = dZ.sum(axis=0)
    dQ = _spmm64_t(rowptr, colidx, vals, dZ)
    dW2 = H1.T @ dQ
    dH1 = dQ @ W2.T
    dpre1 = dH1 * (pre1 > 0.0)
    dW1 = P.T @ dpre1
    db1 = dpre1.sum(axis=0)
    return SimpleNamespace(P=P, pre1=pre1, H1=H1, Q=Q, Z=Z, loss=loss, dZ=dZ, dQ=dQ, dW2=dW2,
                           db2=db2, dH1=dH1, dpre1=dpre1, dW1=dW1, db1=db1)


def gin_step(rowptr, colidx, vals, X, Ws, bs, labels, eps=0.0):
    """L-layer GIN forward + backward in fp64 (paper Sec. 5 "Benchmarks"; Sec. 2.1 aggregate-sum
    followed by the Update).  Layer l: A_l = A.H_l + eps*H_l, pre_l = A_l W_l + b_l,
    H_{l+1} = relu(pre_l) except after the last layer, whose pre-activation is the logits.
    loss = mean softmax cross-entropy.  `vals` None = unit entries.  Returns the logits, the
    loss and the gradient of every W_l and b_l.
    """
    f = np.float64
    Ws = [np.asarray(w, f) for w in Ws]
    bs = [np.asarray(b, f) for b in bs]
    L = len(Ws)
    n = np.asarray(X).shape[0]
    H = [np.asarray(X, f)]
    A, pre = [], []
    for l in range(L):
        a = _spmm64(rowptr, colidx, vals, H[l]) + eps * H[l]
        A.append(a)
        pre.append(a @ Ws[l] + bs[l])
        if l < L - 1:
            H.append(np.maximum(pre[l], 0.0))
    Z = pre[-1]
    zmax = Z.max(axis=1, keepdims=True)
    ez = np.exp(Z - zmax)
    lse = np.log(ez.sum(axis=1)) + zmax[:, 0]
    loss = float(np.mean(lse - Z[np.arange(n), labels]))
    dpre = ez / ez.sum(axis=1, keepdims=True)
    dpre[np.arange(n), labels] -= 1.0
    dpre /= n
    dW, db, dpres = [None] * L, [None] * L, [None] * L
    for l in range(L - 1, -1, -1):
        dpres[l] = dpre
        dW[l] = A[l].T @ dpre
        db[l] = dpre.sum(axis=0)
        if l == 0:
            break
        dA = dpre @ Ws[l].T
        dH = _spmm64_t(rowptr, colidx, vals, dA) + eps * dA
        dpre = dH * (pre[l - 1] > 0.0)
    return SimpleNamespace(Z=Z, loss=loss, dW=dW, db=db, A=A, H=H, pre=pre, dpre=dpres)


def _spmm64(rowptr, colidx, vals, M):
    """A.M for an fp64 right-hand side (plain python/numpy row loop via CSR)."""
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    a = np.ones(colidx.size, np.float64) if vals is None else np.asarray(vals, np.float64)
    contrib = a[:, None] * M[colidx]
    out = np.zeros_like(M, dtype=np.float64)
    rows = np.repeat(np.arange(rowptr.size - 1), np.diff(rowptr))
    np.add.at(out, rows, contrib)
    return out


def _spmm64_t(rowptr, colidx, vals, M):
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    a = np.ones(colidx.size, np.float64) if vals is None else np.asarray(vals, np.float64)
    rows = np.repeat(np.arange(rowptr.size - 1), np.diff(rowptr))
    contrib = a[:, None] * M[rows]
    out = np.zeros_like(M, dtype=np.float64)
    np.add.at(out, colidx, contrib)
    return out
