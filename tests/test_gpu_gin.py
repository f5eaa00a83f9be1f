"""GPU parity of the L-layer GIN training step against the fp64 oracle."""
import math

import numpy as np
import pytest

import oracle
import paper_2305_17408_amd as ag
from ag_inputs import (config_graph, planted_partition, mixed_density, directed_random, features, glorot_uniform,
                       labels)
from gpu_util import say

pytestmark = pytest.mark.gpu


def run_step(g, widths, eps=0.0, seed=0, zero=False, wscale=1.0):
    import torch
    dev = "cuda"
    L = len(widths) - 1
    by_width = {}
    for w in widths:                                    # one plan per distinct width, clones of the first
        if w not in by_width:
            by_width[w] = (ag.ag_plan_clone_for_width(by_width[widths[0]], w) if by_width else
                           ag.ag_plan_create(g.rowptr, g.colidx, g.vals, g.n, w, layout=ag.AG_LAYOUT_REORDERED))
    plans = [by_width[w] for w in widths]
    perm = ag.ag_plan_export(plans[0])["perm"]
    X = features(g.n, widths[0], 10 + seed)
    Ws = [(wscale * glorot_uniform(widths[l], widths[l + 1], 30 + seed + l)).astype(np.float32) for l in range(L)]
    bs = [(0.05 * features(1, widths[l + 1], 50 + seed + l)[0]).astype(np.float32) for l in range(L)]
    if zero:
        Ws, bs = [w * 0 for w in Ws], [b * 0 for b in bs]
    y = labels(g.n, widths[-1], 15 + seed)
    ref = oracle.gin_step(g.rowptr, g.colidx, g.vals, X, Ws, bs, y, eps=eps)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    Xp, yp = t(X[perm]), t(y[perm])
    dW = [torch.full((widths[l], widths[l + 1]), float("nan"), device=dev) for l in range(L)]
    db = [torch.full((widths[l + 1],), float("nan"), device=dev) for l in range(L)]
    loss = torch.empty(1, device=dev)
    logits = torch.empty(g.n, widths[-1], device=dev)
    ws = torch.empty(ag.ag_gin_workspace_bytes(g.n, widths) // 4, device=dev)
    Wd, bd = [t(w) for w in Ws], [t(b) for b in bs]
    for rep in range(2):
        ag.ag_gin_step(plans, widths=widths, eps=eps, W=Wd, b=bd, dW=dW, db=db, loss=loss, logits=logits,
                       X=Xp, labels=yp, workspace=ws)
    torch.cuda.synchronize()
    for p in by_width.values():
        ag.ag_plan_destroy(p)
    got = dict(loss=float(loss.item()), Z=logits.cpu().numpy(), dW=[a.cpu().numpy() for a in dW],
               db=[a.cpu().numpy() for a in db])
    return got, ref, perm


def compare(got, ref, perm):
    """Loss to 1e-5 relative, logits to 1e-4 of their largest value, and every gradient entry to the
    band of the aggregation itself, once per layer of the chain it went through: an entry of dW_l
    or db_l is the end of L chained layer products (l forward, L - l backward), each with its own
    fp32 rounding, so |g - g_ref| <= L * (1e-5 * sum|terms| + 1e-7) with the terms of the last
    contraction (dW_l = A_l^T dpre_l, db_l = column sums of dpre_l) from the oracle's intermediates."""
    assert abs(got["loss"] - ref.loss) <= 1e-5 * abs(ref.loss), (got["loss"], ref.loss)
    np.testing.assert_allclose(got["Z"], ref.Z[perm], rtol=0, atol=1e-4 * np.abs(ref.Z).max())
    L = len(ref.dW)
    for l in range(L):
        S = {"dW": np.abs(ref.A[l]).T @ np.abs(ref.dpre[l]), "db": np.abs(ref.dpre[l]).sum(0)}
        for k, a, r in (("dW", got["dW"][l], ref.dW[l]), ("db", got["db"][l], ref.db[l])):
            ratio = float((np.abs(a - r) / (L * (1e-5 * S[k] + 1e-7))).max())
            say(k, l, "worst err/bound", ratio)
            assert np.isfinite(a).all() and ratio <= 1.0, (k, l, ratio)


# [40, 48, 36, 12] and [64, 32, 24, 10]: transforms of 17 .. 64 output columns with k >= 32 run on the
# register-resident bf16-pieces kernel with work-groups of two / one wavefronts, ragged in k and n
@pytest.mark.parametrize("widths", [[24, 40, 8], [32, 64, 64, 64, 64, 16], [12, 20, 20], [8, 6, 10, 33], [16, 5],
                                    [40, 48, 36, 12], [64, 32, 24, 10]])
def test_gin_step_small(widths):
    # unit weights, mixed densities so the dense kernels take part; the wide-last-layer cases use
    # the aggregate-first order for the last layer, the narrow ones the transform-first order
    g = mixed_density(6, 64, 0.3, 6, 0.05, 5)
    got, ref, perm = run_step(g, widths)
    compare(got, ref, perm)


@pytest.mark.parametrize("n", [1, 7, 33, 130])
@pytest.mark.parametrize("widths", [[32, 64, 64, 16], [40, 48, 36, 12], [64, 32, 1]])
def test_gin_step_tiny_graphs(n, widths):
    # fewer rows than one 32-row block of the transform kernels / a few blocks with a ragged tail;
    # a unit-weight ring with self loops; a single class
    from ag_inputs import from_edges
    u = np.arange(n)
    g = from_edges(n, u, (u + 1) % n)
    got, ref, perm = run_step(g, widths, seed=n)
    compare(got, ref, perm)


def test_gin_step_directed_graph_with_eps():
    g = directed_random(3000, 5.0, 3, weighted=False)          # a missing transpose would show
    got, ref, perm = run_step(g, [16, 32, 32, 4], eps=0.3)
    compare(got, ref, perm)


def test_gin_zero_weights_loss_is_log_classes():
    g = planted_partition(16, 64, 8, 0.7, 5)
    got, ref, perm = run_step(g, [16, 32, 10], zero=True)
    assert abs(got["loss"] - math.log(10.0)) < 1e-5


def test_gin_step_rejects_mismatching_plans():
    import torch
    g = planted_partition(4, 64, 8, 0.7, 5)
    p16 = ag.ag_plan_create(g.rowptr, g.colidx, None, g.n, 16, layout=ag.AG_LAYOUT_REORDERED)
    p8 = ag.ag_plan_clone_for_width(p16, 8)
    other = ag.ag_plan_create(g.rowptr, g.colidx, None, g.n, 8, layout=ag.AG_LAYOUT_REORDERED)
    dev = "cuda"
    W, b = [torch.zeros(16, 8, device=dev)], [torch.zeros(8, device=dev)]
    dW, db = [torch.zeros(16, 8, device=dev)], [torch.zeros(8, device=dev)]
    loss, X = torch.zeros(1, device=dev), torch.zeros(g.n, 16, device=dev)
    y = torch.zeros(g.n, dtype=torch.int32, device=dev)
    ws = torch.empty(ag.ag_gin_workspace_bytes(g.n, [16, 8]) // 4, device=dev)
    kw = dict(widths=[16, 8], eps=0.0, W=W, b=b, dW=dW, db=db, loss=loss, logits=None, X=X, labels=y)
    ag.ag_gin_step([p16, p8], workspace=ws, **kw)                          # fine
    with pytest.raises(RuntimeError):
        ag.ag_gin_step([p16, other], workspace=ws, **kw)                   # another topology object
    with pytest.raises(RuntimeError):
        ag.ag_gin_step([p8, p8], workspace=ws, **kw)                       # wrong width
    with pytest.raises(RuntimeError):
        ag.ag_gin_step([p16, p8], workspace=ws[: ws.numel() // 2], **kw)   # workspace too small
    torch.cuda.synchronize()
    for p in (p16, p8, other):
        ag.ag_plan_destroy(p)


def test_gin_step_config4_scaled():
    # unit weights and sums over ~40 neighbours per layer: the weights are scaled down so that the
    # activations stay O(1) through five layers (unscaled, the logits reach 1e6, where one fp32
    # ulp of a logit already changes the softmax, and no fp32 implementation has stable gradients)
    g = config_graph(4, scale=1 / 32)
    got, ref, perm = run_step(g, [32, 64, 64, 64, 64, 16], wscale=0.05)
    say("loss", got["loss"], ref.loss)
    compare(got, ref, perm)
