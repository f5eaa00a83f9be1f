"""Property test (CPU): on random small matrices and random options the library's host
decomposition equals the oracle's bit for bit, and its invariants hold."""
import numpy as np
from hypothesis import given, settings, strategies as st, HealthCheck

import oracle
import paper_2305_17408_amd as ag
from ag_inputs.graphs import _csr_from_directed


@st.composite
def random_matrix(draw):
    n = draw(st.sampled_from([1, 2, 3, 5, 8, 13, 21, 34, 60, 150, 400]))
    m = draw(st.integers(0, 5 * n))
    seed = draw(st.integers(0, 2 ** 31 - 1))
    rng = np.random.default_rng(seed)
    clustered = draw(st.booleans())
    if clustered and n >= 8:                          # a few planted groups so that blocks appear
        k = draw(st.integers(2, 6))
        grp = rng.integers(0, k, size=n)
        r = rng.integers(0, n, size=m)
        c = np.array([rng.choice(np.flatnonzero(grp == grp[i])) for i in r], dtype=np.int64) if m else np.empty(0, np.int64)
    else:
        r = rng.integers(0, n, size=m)
        c = rng.integers(0, n, size=m)
    if draw(st.booleans()):                           # symmetric pattern
        r, c = np.concatenate([r, c]), np.concatenate([c, r])
    if draw(st.booleans()):                           # diagonal
        d = np.arange(n)
        r, c = np.concatenate([r, d]), np.concatenate([c, d])
    g = _csr_from_directed(n, r.astype(np.int64), c.astype(np.int64))
    if draw(st.booleans()):
        g.vals = rng.uniform(-2, 2, size=g.nnz).astype(np.float32)
    return g


@settings(max_examples=150, deadline=None, suppress_health_check=[HealthCheck.too_slow])
@given(g=random_matrix(), cap=st.integers(1, 256), minb=st.integers(1, 20), sweeps=st.integers(1, 8),
       levels=st.integers(1, 12), order=st.sampled_from([-1, 1, 2, 3]), method=st.sampled_from([0, 1]))
def test_library_equals_oracle(g, cap, minb, sweeps, levels, order, method):
    kw = dict(block_cap=cap, min_block=minb, sweeps=sweeps, max_levels=levels, order_levels=order, method=method)
    p = ag.ag_plan_create(g.rowptr, g.colidx, g.vals, g.n, 4, flags=ag.AG_FLAG_HOST_ONLY, **kw)
    try:
        e = ag.ag_plan_export(p)
        stt = ag.ag_plan_stats(p)
    finally:
        ag.ag_plan_destroy(p)
    r = oracle.reorder(g.rowptr, g.colidx, **dict(kw, order_levels=max(order, 0)))
    assert np.array_equal(e["perm"], r.perm) and np.array_equal(e["iperm"], r.iperm)
    assert np.array_equal(e["blk_ptr"], r.blk_ptr)
    s = oracle.split(g.rowptr, g.colidx, g.vals, r.perm, r.iperm, r.blk_ptr)
    for k in ("intra_rowptr", "intra_col", "inter_rowptr", "inter_col"):
        assert np.array_equal(e[k], getattr(s, k)), k
    if g.vals is not None and g.nnz > 0:                  # (an empty weighted matrix is the same as a unit one)
        assert np.array_equal(e["intra_val"].view(np.uint32), s.intra_val.view(np.uint32))
        assert np.array_equal(e["inter_val"].view(np.uint32), s.inter_val.view(np.uint32))
    # invariants
    sizes = np.diff(e["blk_ptr"])
    assert np.all(sizes >= minb) and np.all(sizes <= cap)
    assert sorted(e["perm"].tolist()) == list(range(g.n))
    assert stt["nnz_intra"] + stt["nnz_inter"] == g.nnz
    assert sum(stt["block_density_hist"]) == stt["n_blocks"]
