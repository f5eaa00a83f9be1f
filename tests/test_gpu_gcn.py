"""GPU parity of the two-layer GCN training step against the fp64 oracle."""
import math

import numpy as np
import pytest

import oracle
import paper_2305_17408_amd as ag
from ag_inputs import config_graph, planted_partition, row_normalise, features, glorot_uniform, labels
from gpu_util import say

pytestmark = pytest.mark.gpu


def run_step(g, fin, hid, ncls, seed=0, zero=False):
    import torch
    dev = "cuda"
    plan_in = ag.ag_plan_create(g.rowptr, g.colidx, g.vals, g.n, fin, layout=ag.AG_LAYOUT_REORDERED)
    plan_out = ag.ag_plan_clone_for_width(plan_in, ncls)
    perm = ag.ag_plan_export(plan_in)["perm"]
    X = features(g.n, fin, 10 + seed)
    W1 = glorot_uniform(fin, hid, 11 + seed)
    W2 = glorot_uniform(hid, ncls, 12 + seed)
    b1 = (0.05 * features(1, hid, 13 + seed)[0]).astype(np.float32)
    b2 = (0.05 * features(1, ncls, 14 + seed)[0]).astype(np.float32)
    if zero:
        W1, W2, b1, b2 = W1 * 0, W2 * 0, b1 * 0, b2 * 0
    y = labels(g.n, ncls, 15 + seed)
    ref = oracle.gcn_step(g.rowptr, g.colidx, g.vals, X, W1, b1, W2, b2, y)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    Xp, yp = t(X[perm]), t(y[perm])                      # plan order
    dW1, db1 = torch.empty(fin, hid, device=dev), torch.empty(hid, device=dev)
    dW2, db2 = torch.empty(hid, ncls, device=dev), torch.empty(ncls, device=dev)
    loss = torch.empty(1, device=dev)
    logits = torch.empty(g.n, ncls, device=dev)
    ws = torch.empty(ag.ag_gcn_workspace_bytes(g.n, fin, hid, ncls) // 4, device=dev)
    for rep in range(2):
        ag.ag_gcn_step(plan_in, plan_out, f_in=fin, hidden=hid, n_class=ncls, W1=t(W1), b1=t(b1), W2=t(W2),
                       b2=t(b2), dW1=dW1, db1=db1, dW2=dW2, db2=db2, loss=loss, logits=logits, X=Xp,
                       labels=yp, workspace=ws)
    torch.cuda.synchronize()
    ag.ag_plan_destroy(plan_out)
    ag.ag_plan_destroy(plan_in)
    got = dict(loss=float(loss.item()), dW1=dW1.cpu().numpy(), db1=db1.cpu().numpy(),
               dW2=dW2.cpu().numpy(), db2=db2.cpu().numpy(), Z=logits.cpu().numpy())
    return got, ref, perm


def compare(got, ref, perm):
    """Loss to 1e-5 relative, logits to 1e-4 of their largest value, and every gradient entry to the
    band of the aggregation itself: |g - g_ref| <= 1e-5 * sum|terms| + 1e-7, the terms being those
    of the contraction that produces the entry (from the oracle's intermediates)."""
    assert abs(got["loss"] - ref.loss) <= 1e-5 * abs(ref.loss), (got["loss"], ref.loss)
    np.testing.assert_allclose(got["Z"], ref.Z[perm], rtol=0, atol=1e-4 * np.abs(ref.Z).max())
    terms = {"dW1": np.abs(ref.P).T @ np.abs(ref.dpre1), "db1": np.abs(ref.dpre1).sum(0),
             "dW2": np.abs(ref.H1).T @ np.abs(ref.dQ), "db2": np.abs(ref.dZ).sum(0)}
    for k, S in terms.items():
        err = np.abs(got[k] - getattr(ref, k))
        ratio = float((err / (1e-5 * S + 1e-7)).max())
        say(k, "max err", err.max(), "worst err/bound", ratio)
        assert np.isfinite(got[k]).all() and ratio <= 1.0, (k, ratio)


def test_gcn_step_small_nonsymmetric():
    g = row_normalise(planted_partition(16, 64, 8, 0.7, 5))      # a missing transpose would show
    got, ref, perm = run_step(g, 24, 40, 8)
    compare(got, ref, perm)


@pytest.mark.parametrize("dims", [(36, 200, 8), (128, 72, 5), (64, 136, 16), (48, 128, 10), (32, 64, 7), (40, 256, 16),
                                  (128, 256, 7), (128, 128, 10), (128, 128, 16), (96, 256, 16), (64, 64, 16), (100, 256, 16), (36, 128, 16), (64, 256, 9)])
def test_gcn_step_ragged_widths(dims):
    # widths that are not multiples of the GEMM tiles (the wide transforms run on bf16 pieces, the
    # narrow ones on fp32 MFMA), hidden widths 64 / 128 / 256 (the backward through the second
    # transform on the matrix instruction) and others (on the vector ALUs), class counts that are
    # not multiples of 4, vertex count not a multiple of 32 or 128; f_in = 128 with hidden 128 / 256
    # takes the LDS-staged fused backward kernel, f_in = 32 / 64 / 96 the register-only one
    g = row_normalise(planted_partition(13, 50, 8, 0.7, 8))
    got, ref, perm = run_step(g, *dims)
    compare(got, ref, perm)


@pytest.mark.parametrize("n", [1, 5, 31, 33, 97])
@pytest.mark.parametrize("dims", [(128, 256, 16), (128, 128, 1), (64, 256, 3), (24, 40, 8)])
def test_gcn_step_tiny_graphs(n, dims):
    # fewer rows than one 32-row block of the fused transform kernels, one block and a bit, a single
    # class (loss 0, all gradients 0 but finite), a ring with self loops
    from ag_inputs import from_edges
    u = np.arange(n)
    g = row_normalise(from_edges(n, u, (u + 1) % n))
    got, ref, perm = run_step(g, *dims, seed=n)
    compare(got, ref, perm)


def test_gcn_step_config3_shape_scaled():
    g = config_graph(3, scale=1 / 64)
    got, ref, perm = run_step(g, 128, 256, 16)
    say("loss", got["loss"], ref.loss)
    compare(got, ref, perm)


def test_gcn_zero_weights_loss_is_log16():
    g = config_graph(3, scale=1 / 256)
    got, ref, perm = run_step(g, 128, 256, 16, zero=True)
    assert abs(got["loss"] - math.log(16.0)) < 1e-5


def test_gcn_step_full_size_config3():
    """The benchmark's GCN workload at full size (N = 1,048,576) against the fp64 oracle.

    With a million vertices the weight gradients are sums of strongly cancelling terms, so they
    are held to the same band as the aggregation itself: |g - g_ref| <= 1e-5 * sum|terms| + 1e-7,
    with sum|terms| taken from the oracle's intermediates."""
    g = config_graph(3)
    say(f"full-size GCN step: n={g.n} nnz={g.nnz}")
    got, ref, perm = run_step(g, 128, 256, 16)
    say("loss", got["loss"], ref.loss)
    compare(got, ref, perm)


def test_gcn_step_replayed_from_a_hip_graph():
    """With both plans' selectors frozen a step only enqueues kernels (no allocation, no host wait,
    no memset nodes), so it can be recorded into a HIP graph: every replay, with eager work and
    synchronisations in between, must reproduce the eager step bit for bit."""
    import torch
    dev = "cuda"
    g = config_graph(3, scale=1 / 64)
    fin, hid, ncls = 128, 256, 16
    plan_in = ag.ag_plan_create(g.rowptr, g.colidx, g.vals, g.n, fin, layout=ag.AG_LAYOUT_REORDERED)
    plan_out = ag.ag_plan_clone_for_width(plan_in, ncls)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    X, y = t(features(g.n, fin, 1)), t(labels(g.n, ncls, 2))
    W1, W2 = t(glorot_uniform(fin, hid, 3)), t(glorot_uniform(hid, ncls, 4))
    b1, b2 = torch.zeros(hid, device=dev), torch.zeros(ncls, device=dev)
    outs = dict(dW1=torch.empty(fin, hid, device=dev), db1=torch.empty(hid, device=dev),
                dW2=torch.empty(hid, ncls, device=dev), db2=torch.empty(ncls, device=dev),
                loss=torch.empty(1, device=dev), logits=torch.empty(g.n, ncls, device=dev))
    ws = torch.empty(ag.ag_gcn_workspace_bytes(g.n, fin, hid, ncls) // 4, device=dev)

    def step(stream=None):
        ag.ag_gcn_step(plan_in, plan_out, f_in=fin, hidden=hid, n_class=ncls, W1=W1, b1=b1, W2=W2, b2=b2, X=X,
                       labels=y, workspace=ws, stream=stream, **outs)

    n = 0
    while n < 200 and not all(ag.ag_plan_selector_info(p, d)["frozen"] for p in (plan_in, plan_out) for d in (0, 1)):
        step()
        n += 1
    say("selectors frozen after", n, "steps")
    step()
    torch.cuda.synchronize()
    eager = {k: v.clone() for k, v in outs.items()}
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step(side)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        for v in outs.values():
            v.fill_(float("nan"))
        ws.fill_(float("nan"))                               # the workspace carries nothing from step to step
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k, v in outs.items():
            assert torch.equal(v, eager[k]), (k, rep)
        step()                                               # eager work between the replays
        torch.cuda.synchronize()
    del graph
    ag.ag_plan_destroy(plan_out)
    ag.ag_plan_destroy(plan_in)
