"""Full-size benchmark workloads: the launch configuration bench.py times (REORDERED layout,
adaptive selector and every forced combination) against the oracle, every element."""
import numpy as np
import pytest

import oracle
import paper_2305_17408_amd as ag
from ag_inputs import config_graph, CONFIGS
from gpu_util import Case, check, say, COMBOS

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("idx", [1, 2, 3, 4])
def test_full_config(idx):
    g = config_graph(idx)
    F = CONFIGS[idx]["F"]
    say(f"config {idx}: n={g.n} nnz={g.nnz} F={F}")
    c = Case(g, F, layout=ag.AG_LAYOUT_REORDERED)
    st = ag.ag_plan_stats(c.plan)
    say({k: st[k] for k in ("n_blocks", "n_block_rows", "n_dense_blocks", "nnz_intra", "nnz_inter",
                             "n_long_rows", "sec_reorder", "sec_split", "sec_build", "sec_upload")})
    # host decomposition bit-exact against the oracle at full size
    r = oracle.reorder(g.rowptr, g.colidx)
    assert np.array_equal(c.exp["perm"], r.perm) and np.array_equal(c.exp["blk_ptr"], r.blk_ptr)
    s = oracle.split(g.rowptr, g.colidx, g.vals, r.perm, r.iperm, r.blk_ptr)
    assert np.array_equal(c.exp["intra_col"], s.intra_col) and np.array_equal(c.exp["inter_col"], s.inter_col)
    assert np.array_equal(c.exp["intra_rowptr"], s.intra_rowptr)
    worst = c.check_all_combos()
    say("worst err/bound", max(worst.values()))
    # adaptive path
    ag.ag_plan_destroy(c.plan)
    c.plan = ag.ag_plan_create(g.rowptr, g.colidx, g.vals, g.n, F, layout=ag.AG_LAYOUT_REORDERED)
    n = 0
    while not ag.ag_plan_selector_info(c.plan, 0)["frozen"] and n < 64:
        y = c.forward()
        n += 1
    check(c.forward(), c.Yref, c.Sy, "adaptive fwd")
    check(c.backward(), c.Dref, c.Sd, "adaptive bwd")
    say("selector", ag.ag_plan_selector_info(c.plan, 0))
    c.close()
