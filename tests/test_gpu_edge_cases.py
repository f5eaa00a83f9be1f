"""More GPU parity cases: paper-faithful community size, odd widths on every kernel family, plans
without blocks, a non-default stream, interleaved plans, single-vertex graphs."""
import numpy as np
import pytest

import oracle
import paper_2305_17408_amd as ag
from ag_inputs import (config_graph, planted_partition, gcn_normalise, mixed_density, from_edges,
                       directed_random, features)
from gpu_util import Case, COMBOS, check, force, say

pytestmark = pytest.mark.gpu


def test_community_size_16_as_in_the_paper():
    g = gcn_normalise(planted_partition(200, 16, 6, 0.8, 71))
    c = Case(g, 32, block_cap=16, min_block=4)
    st = ag.ag_plan_stats(c.plan)
    assert st["n_blocks"] > 150 and st["density_intra"] > 0.2
    c.check_all_combos()
    c.close()


@pytest.mark.parametrize("F", [3, 36, 100, 132, 512, 66, 10])
def test_odd_widths_with_dense_class_blocks(F):
    g = mixed_density(5, 128, 0.35, 5, 0.03, 73)
    c = Case(g, F, seed=F)
    assert ag.ag_plan_stats(c.plan)["n_dense_blocks"] >= 4
    c.check_all_combos(directions=(0,))
    gw = gcn_normalise(g)
    c2 = Case(gw, F, seed=F + 1)
    c2.check_all_combos(combos=["split_dense_narrow", "fused_narrow"], directions=(0,))
    c.close()
    c2.close()


@pytest.mark.parametrize("F", [16, 64, 100, 128, 31])
def test_blocks_of_up_to_256_rows(F):
    # planted communities of 200 and of 256 vertices with block_cap 256: diagonal blocks beyond 128
    # rows (the block-sparse kernel's larger LDS tile, two runs of rows per block), next to a
    # dense-class candidate that has to stay at 128 rows or fewer; weighted and unit, every combination
    import numpy as np
    from ag_inputs import planted_partition, gcn_normalise, mixed_density
    for g in (gcn_normalise(planted_partition(9, 200, 14, 0.85, 21)), planted_partition(5, 256, 30, 0.9, 22)):
        c = Case(g, F, seed=F, block_cap=256, layout=ag.AG_LAYOUT_REORDERED)
        sizes = np.diff(c.exp["blk_ptr"])
        say(f"  F={F} blocks {sizes.tolist()}")
        assert sizes.max() > 128 and sizes.max() <= 256
        c.check_all_combos()
        c.close()
    g = mixed_density(4, 128, 0.3, 6, 0.0, 23)           # isolated dense communities: dense-class blocks (<= 128 rows) under a cap of 256
    c = Case(g, F, seed=F + 1, block_cap=256)
    assert ag.ag_plan_stats(c.plan)["n_dense_blocks"] > 0
    c.check_all_combos()
    c.close()


def test_a_reordering_from_the_caller_with_odd_blocks():
    # a partition handed in by the caller instead of the library's own community detection: planted
    # communities of 90 vertices cut into blocks of 1, 256, 7, 100 and 90 rows (blocks that straddle
    # communities, a one-row block, the largest block), the rest tail; every kernel combination
    g = gcn_normalise(planted_partition(8, 90, 10, 0.7, 31))
    perm = np.arange(g.n, dtype=np.int32)
    blk = np.array([0, 1, 257, 264, 364, 454], np.int32)
    for layout in (ag.AG_LAYOUT_ORIGINAL, ag.AG_LAYOUT_REORDERED):
        c = Case(g, 40, seed=3, layout=layout, reuse=(perm, blk))
        assert np.array_equal(c.exp["blk_ptr"], blk) and np.array_equal(c.exp["perm"], perm)
        c.check_all_combos()
        c.close()
    # the exported reordering of a plan gives the same plan again
    c = Case(g, 40, seed=3)
    c2 = Case(g, 40, seed=3, reuse=(c.exp["perm"].copy(), c.exp["blk_ptr"].copy()))
    assert np.array_equal(c.exp["intra_col"], c2.exp["intra_col"])
    force(c.plan, "fused_narrow", 0)
    force(c2.plan, "fused_narrow", 0)
    assert c.torch.equal(c.forward(), c2.forward())
    c.close()
    c2.close()


def test_no_blocks_at_all_and_tiny_graphs():
    # uniform sparse graph with a high min_block: every vertex lands in the tail
    g = directed_random(4000, 3.0, 79)
    c = Case(g, 24, min_block=129)        # larger than any community can get
    assert ag.ag_plan_stats(c.plan)["n_blocks"] == 0
    c.check_all_combos()
    # adaptive on a block-less plan
    p = ag.ag_plan_create(g.rowptr, g.colidx, g.vals, g.n, 24, min_block=129)
    import torch
    x = torch.from_numpy(c.H).cuda()
    y = torch.empty_like(x)
    for _ in range(48):
        ag.ag_aggregate(p, x, y)
    torch.cuda.synchronize()
    check(y, c.Yref, c.Sy, "adaptive, no blocks")
    assert ag.ag_plan_selector_info(p, 0)["frozen"]
    ag.ag_plan_destroy(p)
    c.close()
    for n in (1, 2, 17):
        g = gcn_normalise(from_edges(n, np.arange(n - 1), np.arange(1, n)))
        c = Case(g, 8, min_block=1)
        c.check_all_combos()
        c.close()


def test_non_default_stream_and_interleaved_plans():
    import torch
    g1 = config_graph(0)
    g2 = gcn_normalise(mixed_density(4, 128, 0.3, 6, 0.02, 83))
    c1, c2 = Case(g1, 16), Case(g2, 48)
    s = torch.cuda.Stream()
    x1, x2 = torch.from_numpy(c1.H).cuda(), torch.from_numpy(c2.H).cuda()
    y1, y2 = torch.empty_like(x1), torch.empty_like(x2)
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        for _ in range(40):                       # through the trials of both plans, interleaved
            ag.ag_aggregate(c1.plan, x1, y1, stream=s)
            ag.ag_aggregate(c2.plan, x2, y2, stream=s)
    s.synchronize()
    check(y1, c1.Yref, c1.Sy, "plan 1 on side stream")
    check(y2, c2.Yref, c2.Sy, "plan 2 on side stream")
    c1.close()
    c2.close()


def test_profiling_api_reports_calls():
    import torch
    c = Case(config_graph(1, scale=1 / 8), 64)
    force(c.plan, "fused_narrow", 0)
    ag.ag_plan_set_profiling(c.plan, True)
    x = torch.from_numpy(c.H).cuda()
    y = torch.empty_like(x)
    for _ in range(70):                           # more than the event ring holds
        ag.ag_aggregate(c.plan, x, y)
    prof = ag.ag_plan_profile(c.plan, 0)
    assert prof["calls"] == 70 and prof["total_ms"] > 0 and prof["compose"] == ag.AG_COMPOSE_FUSED
    assert prof["class_ms"][0] > 0
    ag.ag_plan_set_profiling(c.plan, False)
    check(y, c.Yref, c.Sy, "profiled calls")
    c.close()


def test_misaligned_feature_pointer_is_rejected():
    import torch
    c = Case(config_graph(0), 16)
    buf = torch.zeros(c.g.n * 16 + 4, device="cuda")
    x = buf[1:1 + c.g.n * 16].view(c.g.n, 16)          # 4-byte aligned only
    y = torch.empty(c.g.n, 16, device="cuda")
    with pytest.raises(ag.AdaptGearError) as ei:
        ag.ag_aggregate(c.plan, x, y)
    assert ei.value.code == ag.AG_ERR_INVALID
    c.close()


def test_gcn_step_with_widths_that_are_not_multiples_of_four():
    from test_gpu_gcn import run_step, compare
    g = gcn_normalise(planted_partition(6, 50, 6, 0.7, 91))      # n = 300
    got, ref, perm = run_step(g, 10, 7, 3)
    compare(got, ref, perm)
    got, ref, perm = run_step(g, 12, 5, 8)
    compare(got, ref, perm)


def test_frozen_plan_can_be_captured_in_a_hip_graph():
    """Once the selector is frozen a call only enqueues kernels (no allocation, no host wait), so it
    can be recorded into a HIP graph; every replay must give the eager result."""
    import torch
    g = config_graph(1, scale=1 / 4)
    c = Case(g, 64, layout=ag.AG_LAYOUT_REORDERED)
    x = torch.from_numpy(c.H).cuda()
    xp = torch.empty_like(x)
    ag.ag_permute_rows(c.plan, x, xp, 64, False)
    y = torch.empty_like(x)
    d = torch.empty_like(x)
    for combo in ("fused_narrow", "split_sparse_narrow", "full_csr_wide"):
        force(c.plan, combo, 0)
        force(c.plan, combo, 1)
        ag.ag_aggregate(c.plan, xp, y)                      # eager warm-up (LDS attribute etc.)
        ag.ag_aggregate_t(c.plan, xp, d)
        torch.cuda.synchronize()
        eager_y, eager_d = y.clone(), d.clone()
        graph = torch.cuda.CUDAGraph()
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            with torch.cuda.graph(graph, stream=s):
                ag.ag_aggregate(c.plan, xp, y, stream=s)
                ag.ag_aggregate_t(c.plan, xp, d, stream=s)
        torch.cuda.current_stream().wait_stream(s)
        for rep in range(3):
            y.fill_(float("nan"))
            d.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(y, eager_y) and torch.equal(d, eager_d), (combo, rep)
        yo = torch.empty_like(y)
        ag.ag_permute_rows(c.plan, y, yo, 64, True)
        check(yo, c.Yref, c.Sy, f"graph replay {combo}")
        del graph
    c.close()


def test_infinite_feature_reaches_only_its_neighbours():
    """Padding / masking inside the sparse kernels must never multiply a stranger's feature row by
    zero: an infinite feature value may only show up in rows that really reference it."""
    import torch
    g = gcn_normalise(planted_partition(10, 100, 8, 0.7, 97))
    c = Case(g, 64, block_cap=100)
    j = 123
    H = c.H.copy()
    H[j, :] = np.inf
    rows = np.repeat(np.arange(g.n), np.diff(g.rowptr))
    touched = np.zeros(g.n, bool)
    touched[rows[g.colidx == j]] = True
    Hfin = c.H.copy()
    Hfin[j, :] = 0.0
    Yfin, Sfin = oracle.spmm(g.rowptr, g.colidx, g.vals, Hfin)
    x = torch.from_numpy(H).cuda()
    for name in ("full_csr_narrow", "full_csr_wide", "split_sparse_narrow", "split_sparse_wide", "fused_narrow",
                 "split_sparse_coo"):
        force(c.plan, name, 0)
        y = torch.empty_like(x)
        ag.ag_aggregate(c.plan, x, y)
        torch.cuda.synchronize()
        yn = y.cpu().numpy().astype(np.float64)
        assert np.all(np.isinf(yn[touched])), name                  # a_ij > 0 here: +inf
        assert np.all(np.isfinite(yn[~touched])), name
        err = np.abs(yn[~touched] - Yfin[~touched])
        assert np.all(err <= 1e-5 * Sfin[~touched] + 1e-7), name
    c.close()


def test_bf16_pieces_reproduce_fp32_values_bit_for_bit():
    """The hardware side of the three-piece cut (round-to-nearest conversion, exact remainders):
    with a permutation matrix as the dense-class block, the bf16 matrix kernel must hand every
    feature value back unchanged, bit for bit, whatever its mantissa."""
    import torch
    from ag_inputs import from_edges
    n, F = 256, 64
    rng = np.random.default_rng(11)
    src = np.concatenate([rng.permutation(128), 128 + rng.permutation(128)])
    g = from_edges(n, np.arange(n), src, self_loops=False, symmetric=False)       # row i = e_src[i], unit weights
    assert g.nnz == n and g.vals is None
    mant = rng.integers(0, 1 << 23, size=(n, F), dtype=np.uint32)
    mant[:, :10] = np.array([0x008000, 0x018000, 0x00FFFF, 0x007FFF, 0x008001, 0x7FFFFF, 0x000080, 0x000180,
                             0x0080FF, 0x00807F], np.uint32)                      # ties and extremes of the rounding
    expo = rng.integers(127 - 40, 127 + 40, size=(n, F), dtype=np.uint32)
    sign = rng.integers(0, 2, size=(n, F), dtype=np.uint32)
    H = ((sign << 31) | (expo << 23) | mant).view(np.float32)
    p = ag.ag_plan_create(g.rowptr, g.colidx, None, n, F, dense_density=1e-9,
                          reuse=(np.arange(n, dtype=np.int32), np.array([0, 128, 256], np.int32)))
    assert ag.ag_plan_stats(p)["n_dense_blocks"] == 2
    x = torch.from_numpy(H).cuda()
    for name in ("split_dense_bf16x3", "fused_dense_bf16x3"):
        force(p, name, 0)
        y = torch.full_like(x, float("nan"))
        ag.ag_aggregate(p, x, y)
        torch.cuda.synchronize()
        assert np.array_equal(y.cpu().numpy().view(np.uint32), H[src].view(np.uint32)), name
    ag.ag_plan_destroy(p)
