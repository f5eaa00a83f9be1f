"""ag_aggregate_static (the entry point for callers that cannot allocate) against ag_aggregate.

Graphs with hub rows, so that the long-row kernels and with them the static scratch array are in
use.  Two calls in a row on one GPU, the second with a smaller input (fewer vertices, fewer
segments, narrower features): the array keeps the first call's contents and the second result
must not depend on them.  Compared bit for bit with ag_aggregate under the same pinned kernels
(the kernels are the same and have a fixed summation order) and with the oracle under the
acceptance bound.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _case(scale, F, combo, seed):
    import torch
    import paper_2305_17408_amd as ag
    import oracle
    from ag_inputs import config_graph, features
    from gpu_util import force, check, say
    g = config_graph(2, scale=scale)                  # power-law graph: hub rows far above 96 entries
    say(f"  static-scratch case n={g.n} nnz={g.nnz} F={F} combo={combo}")
    plan = ag.ag_plan_create(g.rowptr, g.colidx, g.vals, g.n, F, layout=ag.AG_LAYOUT_REORDERED)
    st = ag.ag_plan_stats(plan)
    assert st["n_long_segments"] > 0
    force(plan, combo, 0)
    H = features(g.n, F, seed)
    x = torch.from_numpy(H).cuda()
    xp = torch.empty_like(x)
    ag.ag_permute_rows(plan, x, xp, F, False)
    y_ref = torch.full_like(x, float("nan"))
    y_new = torch.full_like(x, float("nan"))
    ag.ag_aggregate(plan, xp, y_ref)
    ag.ag_aggregate_static(plan, xp, y_new)
    torch.cuda.synchronize()
    assert torch.equal(y_ref, y_new), "static-scratch result differs from ag_aggregate"
    out = torch.empty_like(x)
    ag.ag_permute_rows(plan, y_new, out, F, True)
    torch.cuda.synchronize()
    Yr, S = oracle.spmm(g.rowptr, g.colidx, g.vals, H)
    check(out, Yr, S, f"static scratch {combo}")
    ag.ag_plan_destroy(plan)


@pytest.mark.parametrize("combo", ["full_csr_narrow", "split_sparse_narrow", "fused_narrow"])
def test_two_calls_in_a_row_second_smaller(combo):
    _case(0.0625, 64, combo, 11)     # 16 384 vertices
    _case(0.03125, 20, combo, 12)    # 8 192 vertices, narrower rows: a smaller footprint in the same array


def test_refuses_unsettled_choice_and_oversized_scratch():
    import torch
    import paper_2305_17408_amd as ag
    from ag_inputs import config_graph
    from gpu_util import force
    g = config_graph(2, scale=0.0625)
    F = 64
    plan = ag.ag_plan_create(g.rowptr, g.colidx, g.vals, g.n, F, layout=ag.AG_LAYOUT_REORDERED)
    x = torch.zeros(g.n, F, device="cuda")
    y = torch.empty_like(x)
    with pytest.raises(ag.AdaptGearError) as e:       # selector trials still ahead
        ag.ag_aggregate_static(plan, x, y)
    assert e.value.code == ag.AG_ERR_UNSUPPORTED and "settled" in str(e.value)
    ag.ag_plan_destroy(plan)
    # a width at which the segments' partial sums exceed the static array
    small = ag.ag_plan_create(g.rowptr, g.colidx, g.vals, g.n, 4, layout=ag.AG_LAYOUT_REORDERED)
    segs = ag.ag_plan_stats(small)["n_long_segments"]
    ag.ag_plan_destroy(small)
    Fbig = 4 * (ag.AG_STATIC_SCRATCH_BYTES // (16 * max(1, segs)) + 8)
    plan = ag.ag_plan_create(g.rowptr, g.colidx, g.vals, g.n, Fbig, layout=ag.AG_LAYOUT_REORDERED)
    force(plan, "full_csr_narrow", 0)
    x = torch.zeros(g.n, Fbig, device="cuda")
    y = torch.empty_like(x)
    with pytest.raises(ag.AdaptGearError) as e:
        ag.ag_aggregate_static(plan, x, y)
    assert e.value.code == ag.AG_ERR_UNSUPPORTED and "scratch" in str(e.value)
    ag.ag_plan_destroy(plan)
