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


def _int_list(text):
    """'0 0 1..3 7' -> [0, 0, 1, 2, 3, 7]"""
    out = []
    for tok in text.split():
        if ".." in tok:
            a, b = tok.split("..")
            out.extend(range(int(a), int(b) + 1))
        else:
            out.append(int(tok))
    return out


def reorder_trace_cases(path=None):
    """The hand-traced reorder cases of tests/golden/reorder_traces.txt as dicts:
    name, n, edges [(u, v)], options {block_cap, min_block, sweeps, ...}, comm, blk_ptr, perm."""
    import os
    if path is None:
        path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "reorder_traces.txt")
    keymap = {"cap": "block_cap"}
    cases = []
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        name, n, edges, opts, comm, blk, perm = [x.strip() for x in line.split("|")]
        kw = {"order_levels": 0}
        for tok in opts.split():
            k, v = tok.split("=")
            kw[keymap.get(k, k)] = int(v)
        cases.append(dict(name=name, n=int(n), edges=[tuple(map(int, p.split("-"))) for p in edges.split()],
                          options=kw, comm=_int_list(comm), blk_ptr=_int_list(blk), perm=_int_list(perm)))
    return cases


def failing_reorder_traces(reorder_fn):
    """Run every hand-traced case through reorder_fn(rowptr, colidx, **options) (the signature of
    oracle.reorder) and return the names of the cases whose result differs from the trace."""
    from ag_inputs import from_edges
    bad = []
    for c in reorder_trace_cases():
        g = from_edges(c["n"], [a for a, _ in c["edges"]], [b for _, b in c["edges"]])
        r = reorder_fn(g.rowptr, g.colidx, **c["options"])
        if (list(map(int, r.comm)) != c["comm"] or list(map(int, r.blk_ptr)) != c["blk_ptr"]
                or list(map(int, r.perm)) != c["perm"]):
            bad.append(c["name"])
    return bad
