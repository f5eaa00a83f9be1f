"""Small test-side utilities (dense reconstruction etc.).  No method code."""
import numpy as np


def dense_from_csr(rowptr, colidx, vals, n=None):
    n = len(rowptr) - 1 if n is None else n
    A = np.zeros((n, n), dtype=np.float64)
    for i in range(n):
        for e in range(rowptr[i], rowptr[i + 1]):
            A[i, colidx[e]] += 1.0 if vals is None else float(vals[e])
    return A


def csr_rows(rowptr):
    return np.repeat(np.arange(len(rowptr) - 1), np.diff(rowptr))


def tol_ok(y, y_ref, S, rel=1e-5, abs_=1e-7):
    """spec acceptance: |y - y_ref| <= rel * sum|a h| + abs, elementwise."""
    err = np.abs(np.asarray(y, np.float64) - y_ref)
    bound = rel * S + abs_
    bad = err > bound
    return (not bad.any()), float((err / bound).max()) if err.size else 0.0
