"""GPU parity of the max aggregator and its adjoint against the oracle.

The maximum is one of the inputs, so Y is compared bit for bit.  The argmax is unique when no
two neighbours hold the same value (random fp32 features): then it is compared exactly and the
adjoint is compared within the aggregation's tolerance band.  With ties, several argmax answers
are right: the test checks that the answer is a neighbour holding the maximum."""
import numpy as np
import pytest

import oracle
import paper_2305_17408_amd as ag
from ag_inputs import config_graph, planted_partition, directed_random, mixed_density, from_edges, features
from gpu_util import REL, ABS, say

pytestmark = pytest.mark.gpu


def run(g, F, H, G=None):
    import torch
    plan = ag.ag_plan_create(g.rowptr, g.colidx, g.vals, g.n, F, layout=ag.AG_LAYOUT_REORDERED)
    e = ag.ag_plan_export(plan)
    perm, iperm = e["perm"], e["iperm"]
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    Hp = t(H[perm])
    Yp = torch.full_like(Hp, float("nan"))
    argp = torch.full((g.n, F), -7, dtype=torch.int32, device="cuda")
    ag.ag_aggregate_max(plan, Hp, Yp, argp)
    out = {}
    if G is not None:
        dHp = torch.full_like(Hp, float("nan"))
        ag.ag_aggregate_max_t(plan, t(G[perm]), argp, dHp)
        out["dH"] = dHp.cpu().numpy()[iperm]
    torch.cuda.synchronize()
    ag.ag_plan_destroy(plan)
    a = argp.cpu().numpy()[iperm]                        # rows back in the caller's order
    out["arg"] = np.where(a >= 0, perm[np.maximum(a, 0)], -1)   # plan numbering -> caller numbering
    out["Y"] = Yp.cpu().numpy()[iperm]
    return out


@pytest.mark.parametrize("F", [128, 64, 32, 16, 6, 7, 200])
def test_max_forward_and_adjoint_tie_free(F):
    g = planted_partition(24, 64, 8, 0.7, 3)
    H, G = features(g.n, F, 1), features(g.n, F, 2)
    Yref, aref = oracle.spmax(g.rowptr, g.colidx, H)
    Dref, S = oracle.spmax_t(aref, G)
    got = run(g, F, H, G)
    assert np.array_equal(got["Y"].astype(np.float64), Yref)
    assert np.array_equal(got["arg"], aref)
    err = np.abs(got["dH"].astype(np.float64) - Dref)
    assert np.all(err <= REL * S + ABS), float((err / (REL * S + ABS)).max())


def test_max_directed_graph_with_empty_rows_and_hub():
    g0 = directed_random(4000, 4.0, 7, weighted=False, self_loops=False)
    rows = np.repeat(np.arange(g0.n), np.diff(g0.rowptr))
    # one row with 1500 entries (several chunks) on top of the random arcs, arcs stay one-directional
    hub_cols = np.random.default_rng(1).choice(g0.n, 1500, replace=False)
    g = from_edges(g0.n, np.concatenate([rows, np.full(1500, 11)]), np.concatenate([g0.colidx, hub_cols]),
                   self_loops=False, symmetric=False)
    assert (np.diff(g.rowptr) == 0).any()
    H, G = features(g.n, 24, 1), features(g.n, 24, 2)
    Yref, aref = oracle.spmax(g.rowptr, g.colidx, H)
    Dref, S = oracle.spmax_t(aref, G)
    got = run(g, 24, H, G)
    assert np.array_equal(got["Y"].astype(np.float64), Yref)
    assert np.array_equal(got["arg"], aref)
    err = np.abs(got["dH"].astype(np.float64) - Dref)
    assert np.all(err <= REL * S + ABS)


def test_max_with_ties_gives_a_valid_argmax():
    g = mixed_density(4, 64, 0.3, 6, 0.05, 9)
    H = np.random.default_rng(3).integers(0, 4, size=(g.n, 16)).astype(np.float32)    # many equal values
    Yref, _ = oracle.spmax(g.rowptr, g.colidx, H)
    got = run(g, 16, H)
    assert np.array_equal(got["Y"].astype(np.float64), Yref)
    arg = got["arg"]
    assert np.all(arg >= 0)                                              # every row has its self loop
    cols = np.arange(16)[None, :]
    assert np.array_equal(H[arg, cols], got["Y"])                        # the named source holds the maximum
    for i in np.random.default_rng(4).choice(g.n, 64, replace=False):    # ... and is a neighbour
        nb = set(g.colidx[g.rowptr[i]:g.rowptr[i + 1]].tolist())
        assert set(arg[i].tolist()) <= nb


def test_max_rejects_caller_order_plans():
    import torch
    g = planted_partition(4, 64, 8, 0.7, 3)
    plan = ag.ag_plan_create(g.rowptr, g.colidx, None, g.n, 8)           # AG_LAYOUT_ORIGINAL
    x = torch.zeros(g.n, 8, device="cuda")
    with pytest.raises(RuntimeError):
        ag.ag_aggregate_max(plan, x, torch.empty_like(x), None)
    ag.ag_plan_destroy(plan)


def test_max_config2_scaled_power_law():
    g = config_graph(2, scale=1 / 16)
    H, G = features(g.n, 128, 1), features(g.n, 128, 2)
    Yref, aref = oracle.spmax(g.rowptr, g.colidx, H)
    Dref, S = oracle.spmax_t(aref, G)
    got = run(g, 128, H, G)
    say("max degree", int(np.diff(g.rowptr).max()))
    assert np.array_equal(got["Y"].astype(np.float64), Yref)
    assert np.array_equal(got["arg"], aref)
    err = np.abs(got["dH"].astype(np.float64) - Dref)
    assert np.all(err <= REL * S + ABS)


def test_max_full_size_config3():
    """The benchmark graph at full size (N = 1,048,576, F = 128): Y bit for bit, argmax exact,
    adjoint within the aggregation's band.  Among 134 M (row, feature) pairs random fp32 draws do
    tie now and then, so every feature column is a permutation of N distinct values (multiples of
    2^-18 around zero, exact in fp32): the argmax is unique everywhere."""
    g = config_graph(3)
    say(f"full-size max aggregator: n={g.n} nnz={g.nnz}")
    rng = np.random.default_rng(11)
    base = ((np.arange(g.n, dtype=np.float64) - g.n / 2) / 2.0 ** 18).astype(np.float32)
    H = np.stack([base[rng.permutation(g.n)] for _ in range(128)], axis=1)
    G = features(g.n, 128, 2)
    Yref, aref = oracle.spmax(g.rowptr, g.colidx, H)
    Dref, S = oracle.spmax_t(aref, G)
    got = run(g, 128, H, G)
    assert np.array_equal(got["Y"].astype(np.float64), Yref)
    assert np.array_equal(got["arg"], aref)
    err = np.abs(got["dH"].astype(np.float64) - Dref)
    ratio = float((err / (REL * S + ABS)).max())
    say("adjoint worst err/bound", ratio)
    assert ratio <= 1.0
