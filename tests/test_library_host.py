"""CPU-side checks of libadaptgear: it loads, exports every declared symbol, validates its
input, and its host decomposition (reorder + split) is bit-identical to the oracle's."""
import os
import re

import numpy as np
import pytest

import oracle
import paper_2305_17408_amd as ag
from ag_inputs import (config_graph, planted_partition, gcn_normalise, directed_random, mixed_density,
                       from_edges)

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def host_plan(g, F=8, **kw):
    return ag.ag_plan_create(g.rowptr, g.colidx, g.vals, g.n, F, flags=ag.AG_FLAG_HOST_ONLY, **kw)


def test_every_declared_symbol_is_exported():
    text = open(os.path.join(ROOT, "include", "adaptgear.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(ag_[a-z_0-9]+)\s*\(", text))
    assert declared == set(ag.EXPORTS), declared ^ set(ag.EXPORTS)
    L = ag.lib()
    for name in declared:
        assert hasattr(L, name), name


def compare_with_oracle(g, **kw):
    p = host_plan(g, **kw)
    try:
        e = ag.ag_plan_export(p)
        okw = {k: v for k, v in kw.items() if k in ("block_cap", "min_block", "sweeps", "max_levels", "method")}
        if "order_levels" in kw:
            okw["order_levels"] = max(kw["order_levels"], 0)
        r = oracle.reorder(g.rowptr, g.colidx, **okw)
        assert np.array_equal(e["perm"], r.perm)
        assert np.array_equal(e["iperm"], r.iperm)
        assert np.array_equal(e["blk_ptr"], r.blk_ptr)
        s = oracle.split(g.rowptr, g.colidx, g.vals, r.perm, r.iperm, r.blk_ptr)
        assert np.array_equal(e["intra_rowptr"], s.intra_rowptr)
        assert np.array_equal(e["intra_col"], s.intra_col)
        assert np.array_equal(e["inter_rowptr"], s.inter_rowptr)
        assert np.array_equal(e["inter_col"], s.inter_col)
        if g.vals is not None:
            assert np.array_equal(e["intra_val"].view(np.uint32), s.intra_val.view(np.uint32))
            assert np.array_equal(e["inter_val"].view(np.uint32), s.inter_val.view(np.uint32))
        else:
            assert e["intra_val"] is None and e["inter_val"] is None
        return ag.ag_plan_stats(p)
    finally:
        ag.ag_plan_destroy(p)


def test_decomposition_bit_exact_config0_and_1():
    st = compare_with_oracle(config_graph(0))
    assert st["symmetric"] == 1 and st["unit_weights"] == 0 and st["nnz"] == 36864
    st = compare_with_oracle(config_graph(1))
    assert st["nnz_intra"] + st["nnz_inter"] == st["nnz"]
    assert st["density_intra"] > 20 * st["density_inter"]      # cf. the paper's density figure


@pytest.mark.parametrize("cfg,scale", [(2, 1 / 16), (3, 1 / 32), (4, 1 / 32)])
def test_decomposition_bit_exact_scaled_configs(cfg, scale):
    compare_with_oracle(config_graph(cfg, scale=scale))


def test_decomposition_bit_exact_directed_and_small_caps():
    st = compare_with_oracle(directed_random(3000, 4.0, 7), min_block=4)
    assert st["symmetric"] == 0
    compare_with_oracle(gcn_normalise(planted_partition(40, 16, 6, 0.8, 3)), block_cap=16, min_block=4)
    compare_with_oracle(planted_partition(10, 100, 10, 0.9, 5), block_cap=100, min_block=1)
    compare_with_oracle(from_edges(50, np.empty(0, int), np.empty(0, int)))
    compare_with_oracle(from_edges(0, np.empty(0, int), np.empty(0, int)))
    compare_with_oracle(config_graph(2, scale=1 / 32), order_levels=-1)         # plain id order
    compare_with_oracle(config_graph(2, scale=1 / 32), order_levels=1)


@pytest.mark.parametrize("cfg,scale", [(0, 1.0), (1, 1.0), (2, 1 / 16), (3, 1 / 32), (4, 1 / 32)])
def test_modularity_gain_method_bit_exact_and_finds_communities(cfg, scale):
    # the second community detection (Sec. 4.2: the partitioner is the user's choice)
    g = config_graph(cfg, scale=scale)
    st = compare_with_oracle(g, method=ag.AG_METHOD_MODULARITY)
    assert st["n_blocks"] > 0 and st["nnz_intra"] + st["nnz_inter"] == st["nnz"]
    if cfg in (0, 1, 3):
        # planted partitions: well over half of the planted intra-community edges end up in blocks
        got = (st["nnz_intra"] - st["n_block_rows"]) / 2 / g.meta["edges"]
        assert got > 0.6 * g.meta["planted_intra_frac"], got
    compare_with_oracle(directed_random(2000, 3.0, 9), method=ag.AG_METHOD_MODULARITY, min_block=4)
    compare_with_oracle(g, method=ag.AG_METHOD_MODULARITY, block_cap=16, order_levels=-1)


def test_number_of_communities_parameter():
    g = gcn_normalise(planted_partition(50, 32, 6, 0.8, 9))          # n = 1600
    p = ag.ag_plan_create(g.rowptr, g.colidx, g.vals, g.n, 4, flags=ag.AG_FLAG_HOST_ONLY, num_communities=50)
    e = ag.ag_plan_export(p)
    ag.ag_plan_destroy(p)
    r = oracle.reorder(g.rowptr, g.colidx, block_cap=32, min_block=16)   # cap = ceil(1600 / 50)
    assert np.array_equal(e["perm"], r.perm) and np.array_equal(e["blk_ptr"], r.blk_ptr)
    assert np.diff(e["blk_ptr"]).max() <= 32


def test_dense_blocks_are_classified():
    g = mixed_density(8, 128, 0.3, 6, 0.02, 11)
    p = host_plan(g)
    st = ag.ag_plan_stats(p)
    ag.ag_plan_destroy(p)
    assert 6 <= st["n_dense_blocks"] <= 9
    assert sum(st["block_density_hist"]) == st["n_blocks"] and sum(st["block_density_hist"][2:]) >= 6
    assert 0.1 < st["density_intra"] < 0.35


def test_factored_values_are_checked_and_leave_the_decomposition_unchanged():
    from ag_inputs import row_normalise
    g = gcn_normalise(mixed_density(6, 96, 0.4, 5, 0.05, 29))
    st = compare_with_oracle(g, block_cap=96, row_scale=g.meta["row_scale"], col_scale=g.meta["col_scale"])
    assert st["factored"] == 1 and st["unit_weights"] == 0
    plain = compare_with_oracle(g, block_cap=96)
    assert plain["factored"] == 0
    # value-free dense kernels come in at a lower density than the ones that read a value tile
    assert st["n_dense_blocks"] >= plain["n_dense_blocks"]
    gm = row_normalise(mixed_density(4, 64, 0.4, 5, 0.05, 31))          # row factors only
    assert compare_with_oracle(gm, block_cap=64, row_scale=gm.meta["row_scale"])["factored"] == 1
    bad = g.meta["row_scale"].copy()
    bad[int(np.argmax(np.diff(g.rowptr)))] *= 1.01                      # a vertex inside a dense community
    with pytest.raises(RuntimeError):
        host_plan(g, row_scale=bad, col_scale=g.meta["col_scale"])
    with pytest.raises(RuntimeError):                                   # factors describe values: vals needed
        ag.ag_plan_create(g.rowptr, g.colidx, None, g.n, 8, row_scale=bad, flags=ag.AG_FLAG_HOST_ONLY)
    with pytest.raises(ValueError):
        host_plan(g, row_scale=bad[:-1])


def test_unsorted_rows_are_sorted_and_values_follow():
    g = gcn_normalise(planted_partition(6, 32, 5, 0.7, 8))
    rng = np.random.default_rng(0)
    col, val = g.colidx.copy(), g.vals.copy()
    for i in range(g.n):
        b, e = g.rowptr[i], g.rowptr[i + 1]
        o = rng.permutation(e - b)
        col[b:e], val[b:e] = col[b:e][o], val[b:e][o]
    p1, p2 = host_plan(g), ag.ag_plan_create(g.rowptr, col, val, g.n, 8, flags=ag.AG_FLAG_HOST_ONLY)
    e1, e2 = ag.ag_plan_export(p1), ag.ag_plan_export(p2)
    for k in e1:
        assert np.array_equal(e1[k], e2[k]), k
    ag.ag_plan_destroy(p1)
    ag.ag_plan_destroy(p2)


def test_a_saved_reordering_is_reused_and_a_foreign_one_is_split_like_the_oracle_does():
    """A plan built from an exported (perm, blk_ptr) equals the plan they came from without running
    the community detection; a partition of the caller's own (any permutation, any block sizes
    up to 256) is decomposed exactly as the oracle's split decomposes it."""
    g = gcn_normalise(planted_partition(20, 48, 6, 0.6, 4))
    p = host_plan(g)
    e = ag.ag_plan_export(p)
    perm, blk = e["perm"].copy(), e["blk_ptr"].copy()
    ag.ag_plan_destroy(p)
    q = host_plan(g, reuse=(perm, blk))
    try:
        f = ag.ag_plan_export(q)
        for k in ("perm", "iperm", "blk_ptr", "intra_rowptr", "intra_col", "inter_rowptr", "inter_col"):
            assert np.array_equal(e[k], f[k]), k
        assert np.array_equal(e["intra_val"].view(np.uint32), f["intra_val"].view(np.uint32))
    finally:
        ag.ag_plan_destroy(q)
    # a foreign partition: rows in reverse order, blocks of 1, 256, 7 and 100 rows, the rest tail
    rng = np.random.default_rng(5)
    perm2 = np.arange(g.n, dtype=np.int32)[::-1].copy()
    rng.shuffle(perm2[300:])
    blk2 = np.array([0, 1, 257, 264, 364], np.int32)
    iperm2 = np.empty_like(perm2)
    iperm2[perm2] = np.arange(g.n, dtype=np.int32)
    q = host_plan(g, reuse=(perm2, blk2))
    try:
        f = ag.ag_plan_export(q)
        s = oracle.split(g.rowptr, g.colidx, g.vals, perm2, iperm2, blk2)
        assert np.array_equal(f["perm"], perm2) and np.array_equal(f["iperm"], iperm2) and np.array_equal(f["blk_ptr"], blk2)
        assert np.array_equal(f["intra_rowptr"], s.intra_rowptr) and np.array_equal(f["intra_col"], s.intra_col)
        assert np.array_equal(f["inter_rowptr"], s.inter_rowptr) and np.array_equal(f["inter_col"], s.inter_col)
        assert np.array_equal(f["intra_val"].view(np.uint32), s.intra_val.view(np.uint32))
        assert np.array_equal(f["inter_val"].view(np.uint32), s.inter_val.view(np.uint32))
    finally:
        ag.ag_plan_destroy(q)
    # no blocks at all: everything is tail
    q = host_plan(g, reuse=(np.arange(g.n, dtype=np.int32), np.zeros(1, np.int32)))
    st = ag.ag_plan_stats(q)
    assert st["n_blocks"] == 0 and st["nnz_intra"] == 0 and st["nnz_inter"] == g.nnz
    ag.ag_plan_destroy(q)


def test_a_broken_saved_reordering_is_refused():
    g = planted_partition(4, 40, 6, 0.6, 2)
    ident = np.arange(g.n, dtype=np.int32)
    ok_blk = np.array([0, 40, 80], np.int32)
    dup = ident.copy(); dup[3] = dup[2]
    neg = ident.copy(); neg[0] = -1
    big = ident.copy(); big[5] = g.n
    for perm, blk in [(dup, ok_blk), (neg, ok_blk), (big, ok_blk),
                      (ident, np.array([1, 40], np.int32)),          # does not start at 0
                      (ident, np.array([0, 40, 40], np.int32)),      # empty block
                      (ident, np.array([0, 80, 40], np.int32)),      # descending
                      (ident, np.array([0, 100, g.n + 1], np.int32))]:  # beyond n
        expect_error(ag.AG_ERR_INVALID, lambda: host_plan(g, reuse=(perm, blk)))
    g2 = planted_partition(3, 100, 6, 0.6, 2)
    expect_error(ag.AG_ERR_INVALID, lambda: host_plan(g2, reuse=(np.arange(g2.n, dtype=np.int32), np.array([0, 257], np.int32))))


def expect_error(code, fn):
    with pytest.raises(ag.AdaptGearError) as ei:
        fn()
    assert ei.value.code == code, ei.value


def test_input_validation():
    g = planted_partition(2, 16, 4, 0.7, 1)
    rp, ci = g.rowptr.copy(), g.colidx.copy()
    bad = ci.copy(); bad[3] = g.n
    expect_error(ag.AG_ERR_INVALID, lambda: ag.ag_plan_create(rp, bad, None, g.n, 4, flags=1))
    bad = ci.copy(); bad[0] = -1
    expect_error(ag.AG_ERR_INVALID, lambda: ag.ag_plan_create(rp, bad, None, g.n, 4, flags=1))
    bad = rp.copy(); bad[5] = bad[4] - 1
    expect_error(ag.AG_ERR_INVALID, lambda: ag.ag_plan_create(bad, ci, None, g.n, 4, flags=1))
    dup = ci.copy(); dup[rp[1] - 1] = dup[rp[1] - 2] if rp[1] - rp[0] >= 2 else dup[0]
    if rp[1] - rp[0] >= 2:
        expect_error(ag.AG_ERR_INVALID, lambda: ag.ag_plan_create(rp, dup, None, g.n, 4, flags=1))
    expect_error(ag.AG_ERR_INVALID, lambda: ag.ag_plan_create(rp, ci, None, g.n + 1, 4, flags=1))
    expect_error(ag.AG_ERR_INVALID, lambda: ag.ag_plan_create(rp, ci, None, g.n, 0, flags=1))
    expect_error(ag.AG_ERR_INVALID, lambda: ag.ag_plan_create(rp, ci, None, g.n, 4, flags=1, block_cap=257))
    expect_error(ag.AG_ERR_INVALID, lambda: ag.ag_plan_create(rp, ci, None, g.n, 4, flags=1, method=2))
    expect_error(ag.AG_ERR_INVALID, lambda: ag.ag_plan_create(rp, ci, None, g.n, 4, flags=1, trials=16))
    p = host_plan(g)
    expect_error(ag.AG_ERR_UNSUPPORTED, lambda: ag.ag_plan_force_kernels(p, ag.AG_CLS_BLOCKS_SPARSE, 0, 1))
    expect_error(ag.AG_ERR_INVALID, lambda: ag.ag_plan_force_kernels(p, 7, 0, 0))
    ag.ag_plan_force_kernels(p, ag.AG_CLS_COMPOSE, ag.AG_DIR_FWD, ag.AG_COMPOSE_FUSED)
    ag.ag_plan_destroy(p)


def test_failing_allocator_callback_gives_nomem_without_touching_the_gpu():
    import ctypes as C
    calls = []
    ALLOC = C.CFUNCTYPE(C.c_void_p, C.c_size_t, C.c_void_p)
    FREE = C.CFUNCTYPE(None, C.c_void_p, C.c_void_p)

    def alloc(nbytes, user):
        calls.append(nbytes)
        return None                                   # always out of memory

    def free(ptr, user):
        calls.append(-1)

    a, f = ALLOC(alloc), FREE(free)
    g = planted_partition(2, 16, 4, 0.7, 1)
    expect_error(ag.AG_ERR_NOMEM, lambda: ag.ag_plan_create(
        g.rowptr, g.colidx, None, g.n, 4, dev_alloc=C.cast(a, C.c_void_p), dev_free=C.cast(f, C.c_void_p)))
    assert calls and calls[0] > 0 and -1 not in calls
    # only one of the two callbacks given is an error
    expect_error(ag.AG_ERR_INVALID, lambda: ag.ag_plan_create(
        g.rowptr, g.colidx, None, g.n, 4, dev_alloc=C.cast(a, C.c_void_p)))


def test_null_and_mismatched_arguments_to_the_drivers():
    g = planted_partition(2, 16, 4, 0.7, 1)
    p = host_plan(g, F=4)
    L = ag.lib()
    assert L.ag_aggregate(p, None, None, None) == ag.AG_ERR_UNSUPPORTED      # host-only plan
    assert L.ag_aggregate(None, None, None, None) == ag.AG_ERR_INVALID
    assert L.ag_plan_stats(None, None) == ag.AG_ERR_INVALID
    assert ag.ag_gcn_workspace_bytes(100, 8, 0, 4) == 0
    assert ag.ag_gcn_workspace_bytes(100, 8, 16, 4) >= 4 * 100 * (8 + 2 * 16 + 4 * 4 + 1)
    ag.ag_plan_destroy(p)
