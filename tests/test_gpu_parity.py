"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle on the same
seeded inputs.  Integer outputs (permutation, split) are compared bit-exactly in
test_library_host.py (host code); here the fp32 results must satisfy
|y - y_ref| <= 1e-5 * sum_j |a_ij h_jk| + 1e-7 for every element, for every kernel combination."""
import numpy as np
import pytest

import oracle
import paper_2305_17408_amd as ag
from ag_inputs import (config_graph, planted_partition, gcn_normalise, row_normalise, directed_random,
                       mixed_density, from_edges, features)
from gpu_util import Case, COMBOS, DETERMINISTIC, check, force, say, usable

pytestmark = pytest.mark.gpu


def test_config0_all_kernel_combinations():
    c = Case(config_graph(0), 16)
    worst = c.check_all_combos()
    say("config0 worst err/bound:", max(worst.values()))
    c.close()


@pytest.mark.parametrize("F", [4, 16, 32, 64, 128, 20, 7, 200, 256, 1, 2, 6, 50, 66, 130, 258])
def test_feature_widths(F):
    g = gcn_normalise(planted_partition(12, 100, 9, 0.7, 31))     # blocks of ~100: ragged tiles
    c = Case(g, F, seed=F, block_cap=100)
    c.check_all_combos(directions=(0,))
    c.close()


def test_reordered_layout_matches():
    g = config_graph(1, scale=1 / 8)
    c = Case(g, 64, layout=ag.AG_LAYOUT_REORDERED)
    c.check_all_combos()
    c.close()


def test_nonsymmetric_backward_uses_the_transpose():
    g = row_normalise(planted_partition(20, 64, 8, 0.75, 13))
    c = Case(g, 32, block_cap=64)
    st = ag.ag_plan_stats(c.plan)
    assert st["symmetric"] == 0
    c.check_all_combos()
    c.close()
    g = directed_random(5000, 6.0, 17)
    c = Case(g, 48, min_block=4)
    c.check_all_combos()
    c.close()


def test_dense_class_blocks_unit_and_weighted():
    g = mixed_density(12, 128, 0.3, 6, 0.02, 23)
    c = Case(g, 32)
    st = ag.ag_plan_stats(c.plan)
    assert st["n_dense_blocks"] >= 10
    c.check_all_combos()
    c.close()
    gw = gcn_normalise(mixed_density(6, 96, 0.4, 5, 0.05, 29))
    for F in (32, 64, 128, 24):
        c = Case(gw, F, block_cap=96)
        assert ag.ag_plan_stats(c.plan)["n_dense_blocks"] >= 4
        c.check_all_combos(combos=["split_dense_narrow", "split_sparse_narrow"])
        with pytest.raises(RuntimeError):            # the bf16 form has no weighted variant
            ag.ag_plan_force_kernels(c.plan, ag.AG_CLS_BLOCKS_DENSE, 0, ag.AG_K_BLOCK_DENSE_BF16X3)
        c.close()
    # unit weights at several widths (two 32-feature tiles, a ragged one, odd widths), ragged blocks
    gu = mixed_density(6, 96, 0.4, 5, 0.05, 31)
    for F in (64, 128, 24, 66, 7):
        c = Case(gu, F, block_cap=96)
        c.check_all_combos(combos=["split_dense_narrow", "split_dense_bf16x3"])
        c.close()
    # magnitudes spread over 12 decades and all 24 mantissa bits in use: the three bf16 pieces
    # must reproduce every feature value exactly for the fp32 bound to hold
    c = Case(gu, 32, block_cap=96)
    rng = np.random.default_rng(77)
    c.H = (c.H * (1.0 + 2.0 ** -23) * 10.0 ** rng.integers(-6, 7, size=c.H.shape)).astype(np.float32)
    c.Yref, c.Sy = oracle.spmm(gu.rowptr, gu.colidx, gu.vals, c.H)
    c.check_all_combos(combos=["split_dense_narrow", "split_dense_bf16x3"], directions=(0,))
    c.close()


def test_fused_dense_kernels_with_many_blocks():
    """From AG_MIN_BLOCKS_OWN_LAUNCH dense-class blocks on, the fused composition runs the dense
    kernels with the remainder epilogue.  One hub vertex inside a dense community gets 400 extra
    neighbours, so its remainder row exceeds the long-row threshold and goes through the
    segment kernels instead of the epilogue."""
    g0 = mixed_density(272, 40, 0.45, 5, 0.05, 37)
    rows = np.repeat(np.arange(g0.n), np.diff(g0.rowptr))
    hub = int(np.argmax(np.diff(g0.rowptr)))
    extra = np.random.default_rng(5).choice(g0.n, 400, replace=False)
    gu = from_edges(g0.n, np.concatenate([rows, np.full(400, hub)]), np.concatenate([g0.colidx, extra]))
    for g, combos, widths in ((gu, ["fused_dense", "fused_dense_bf16x3", "fused_narrow"], (32, 64, 128, 24, 66, 7)),
                              (gcn_normalise(gu), ["fused_dense", "fused_narrow"], (32, 128, 24))):
        for F in widths:
            c = Case(g, F, block_cap=40)
            st = ag.ag_plan_stats(c.plan)
            assert st["n_dense_blocks"] >= ag.AG_MIN_BLOCKS_OWN_LAUNCH, st["n_dense_blocks"]
            assert st["n_long_rows"] >= 1 and c.exp["iperm"][hub] < c.exp["blk_ptr"][-1]
            c.check_all_combos(combos=combos)
            c.close()


def test_factored_values_value_free_blocks():
    """With row_scale / col_scale the diagonal blocks run without stored values (pattern kernels,
    the bf16 dense form included); results must still match the oracle, which uses the values."""
    # symmetric GCN normalisation on a graph with dense communities, several widths, ragged blocks
    gw = gcn_normalise(mixed_density(6, 96, 0.4, 5, 0.05, 29))
    for F in (32, 64, 128, 24, 7):
        c = Case(gw, F, block_cap=96, factored=True)
        st = ag.ag_plan_stats(c.plan)
        assert st["factored"] == 1 and st["n_dense_blocks"] >= 4
        c.check_all_combos()
        c.close()
    # aggregate-mean: row factors only, non-symmetric matrix, so the backward swaps the roles
    gm = row_normalise(mixed_density(6, 64, 0.4, 5, 0.05, 31))
    for F in (32, 20):
        c = Case(gm, F, block_cap=64, factored=True)
        assert ag.ag_plan_stats(c.plan)["symmetric"] == 0
        c.check_all_combos()
        c.close()
    # sparse communities (no dense class) and the fused composition at config-3 shape
    c = Case(config_graph(3, scale=1 / 64), 128, factored=True, layout=ag.AG_LAYOUT_REORDERED)
    c.check_all_combos()
    c.close()
    # many dense-class blocks: the fused dense kernels with scales
    g0 = mixed_density(272, 40, 0.45, 5, 0.05, 37)
    c = Case(gcn_normalise(g0), 32, block_cap=40, factored=True)
    assert ag.ag_plan_stats(c.plan)["n_dense_blocks"] >= ag.AG_MIN_BLOCKS_OWN_LAUNCH
    c.check_all_combos(combos=["fused_dense", "fused_dense_bf16x3", "fused_narrow", "split_dense_bf16x3"])
    c.close()
    # factors that do not reproduce the values are refused
    bad = gw.meta["row_scale"].copy()
    bad[5] *= 1.01
    with pytest.raises(RuntimeError):
        ag.ag_plan_create(gw.rowptr, gw.colidx, gw.vals, gw.n, 8, row_scale=bad, col_scale=gw.meta["col_scale"],
                          flags=ag.AG_FLAG_HOST_ONLY)
    with pytest.raises(RuntimeError):                    # factors need values
        ag.ag_plan_create(gw.rowptr, gw.colidx, None, gw.n, 8, row_scale=bad, flags=ag.AG_FLAG_HOST_ONLY)


def test_power_law_long_rows():
    g = config_graph(2, scale=1 / 16)
    c = Case(g, 128)
    st = ag.ag_plan_stats(c.plan)
    assert st["n_long_rows"] > 10 and st["n_long_segments"] > st["n_long_rows"]
    c.check_all_combos()
    c.close()
    # one hub connected to everything: a single row of 6000 entries, everything else short
    n = 6000
    g = gcn_normalise(from_edges(n, np.zeros(n - 1, int), np.arange(1, n)))
    for F in (16, 128):
        c = Case(g, F)
        c.check_all_combos()
        c.close()


def test_exact_cases():
    import torch
    # identity matrix: Y == H bit for bit
    n = 300
    g = gcn_normalise(from_edges(n, np.empty(0, int), np.empty(0, int)))
    c = Case(g, 16)
    for name in COMBOS:
        if not usable(name, g):
            continue
        force(c.plan, name, 0)
        y = c.forward().cpu().numpy()
        assert np.array_equal(y, c.H), name
    c.close()
    # unit weights and all-ones features: integer degree sums, exact in fp32 in any order
    g = mixed_density(6, 128, 0.3, 6, 0.02, 41)
    c = Case(g, 32)
    ones = torch.ones(g.n, 32, device="cuda")
    deg = np.diff(g.rowptr).astype(np.float32)
    for name in COMBOS:
        force(c.plan, name, 0)
        y = torch.empty_like(ones)
        ag.ag_aggregate(c.plan, ones, y)
        torch.cuda.synchronize()
        assert np.array_equal(y.cpu().numpy(), np.tile(deg[:, None], (1, 32))), name
    c.close()


def test_symmetric_matrix_backward_is_the_forward_kernel():
    c = Case(config_graph(0), 16)
    assert ag.ag_plan_stats(c.plan)["symmetric"] == 1
    for name in DETERMINISTIC:
        if not usable(name, c.g):
            continue
        force(c.plan, name, 0)
        force(c.plan, name, 1)
        c.G = c.H                                   # same input both ways
        assert np.array_equal(c.forward().cpu().numpy(), c.backward().cpu().numpy()), name
    c.close()


def test_runs_are_bitwise_reproducible():
    g = config_graph(2, scale=1 / 32)
    c = Case(g, 64)
    for name in DETERMINISTIC:
        if not usable(name, c.g):
            continue
        force(c.plan, name, 0)
        a = c.forward().cpu().numpy()
        b = c.forward().cpu().numpy()
        assert np.array_equal(a, b), name
    c.close()


def test_degenerate_inputs():
    import torch
    # no vertices
    p = ag.ag_plan_create(np.zeros(1, np.int32), np.empty(0, np.int32), None, 0, 8)
    x = torch.empty(0, 8, device="cuda")
    y = torch.empty(0, 8, device="cuda")
    ag.ag_aggregate(p, x, y)
    ag.ag_plan_destroy(p)
    # rows without any entry give zeros (also inside blocks)
    g = planted_partition(4, 32, 6, 0.8, 3)
    rp = g.rowptr.astype(np.int64).copy()
    keep = np.ones(g.nnz, bool)
    for i in (0, 5, 77):
        keep[rp[i]:rp[i + 1]] = False
    rows = np.repeat(np.arange(g.n), np.diff(g.rowptr))[keep]
    from ag_inputs.graphs import _csr_from_directed
    g2 = _csr_from_directed(g.n, rows.astype(np.int64), g.colidx[keep].astype(np.int64))
    c = Case(g2, 16, min_block=8, block_cap=32)
    c.check_all_combos()
    c.close()
    # error paths never launch anything
    c = Case(planted_partition(2, 16, 4, 0.7, 1), 8)
    h = torch.zeros(32, 8, device="cuda")
    with pytest.raises(ag.AdaptGearError):
        ag.ag_aggregate(c.plan, h, h)                       # aliasing
    c.close()


def test_adaptive_selector_freezes_and_stays_correct():
    g = mixed_density(16, 128, 0.3, 6, 0.02, 53)
    c = Case(g, 32, trials=2)
    calls = 0
    while not ag.ag_plan_selector_info(c.plan, 0)["frozen"]:
        check(c.forward(), c.Yref, c.Sy, f"trial call {calls}")
        calls += 1
        assert calls < 64
    info = ag.ag_plan_selector_info(c.plan, 0)
    say("selector:", info)
    assert info["choice"][ag.AG_CLS_COMPOSE] in (0, 1, 2, 3)
    assert info["choice"][ag.AG_CLS_BLOCKS_DENSE] in (0, 1, 2)
    assert info["choice"][ag.AG_CLS_REMAINDER] in (0, 1, 2)
    check(c.forward(), c.Yref, c.Sy, "after freeze")
    # backward has its own state
    assert not ag.ag_plan_selector_info(c.plan, 1)["frozen"]
    check(c.backward(), c.Dref, c.Sd, "bwd trial")
    c.close()


def test_clone_for_width_shares_topology():
    import torch
    g = config_graph(0)
    c = Case(g, 16)
    p2 = ag.ag_plan_clone_for_width(c.plan, 40)
    H = features(g.n, 40, 5)
    Yref, S = oracle.spmm(g.rowptr, g.colidx, g.vals, H)
    x = torch.from_numpy(H).cuda()
    y = torch.empty_like(x)
    for _ in range(3):
        ag.ag_aggregate(p2, x, y)
    torch.cuda.synchronize()
    check(y, Yref, S, "clone F=40")
    ag.ag_plan_destroy(p2)
    check(c.forward(), c.Yref, c.Sy, "original after clone destroyed")
    c.close()


def test_gin_layer_with_eps():
    import torch
    g = config_graph(4, scale=1 / 128)
    c = Case(g, 32)
    x = torch.from_numpy(c.H).cuda()
    y = torch.empty_like(x)
    eps = 0.25
    ag.ag_gin_layer(c.plan, eps, x, y)
    torch.cuda.synchronize()
    ref = c.Yref + eps * c.H.astype(np.float64)
    check(y, ref, c.Sy + abs(eps) * np.abs(c.H), "gin eps")
    ag.ag_gin_layer_t(c.plan, 0.0, x, y)
    torch.cuda.synchronize()
    Dref, Sd = oracle.spmm_t(g.rowptr, g.colidx, None, c.H)
    check(y, Dref, Sd, "gin bwd")
    c.close()
