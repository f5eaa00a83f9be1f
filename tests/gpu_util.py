"""Helpers for the GPU parity tests: run the HIP path through the C ABI binding and compare it
with the CPU oracle under the acceptance bound |y - y_ref| <= 1e-5 * sum|a h| + 1e-7."""
import sys

import numpy as np

import oracle
import paper_2305_17408_amd as ag

REL, ABS = 1e-5, 1e-7

COMBOS = {
    # name: (compose, dense-class kernel, remainder kernel)
    "full_csr_narrow": (ag.AG_COMPOSE_FULL_CSR, ag.AG_K_BLOCK_SPARSE, ag.AG_K_CSR_NARROW),
    "full_csr_wide": (ag.AG_COMPOSE_FULL_CSR_WIDE, ag.AG_K_BLOCK_SPARSE, ag.AG_K_CSR_WIDE),
    "split_sparse_narrow": (ag.AG_COMPOSE_SPLIT, ag.AG_K_BLOCK_SPARSE, ag.AG_K_CSR_NARROW),
    "split_sparse_wide": (ag.AG_COMPOSE_SPLIT, ag.AG_K_BLOCK_SPARSE, ag.AG_K_CSR_WIDE),
    "split_dense_narrow": (ag.AG_COMPOSE_SPLIT, ag.AG_K_BLOCK_DENSE, ag.AG_K_CSR_NARROW),
    "split_dense_bf16x3": (ag.AG_COMPOSE_SPLIT, ag.AG_K_BLOCK_DENSE_BF16X3, ag.AG_K_CSR_NARROW),
    "fused_dense": (ag.AG_COMPOSE_FUSED, ag.AG_K_BLOCK_DENSE, ag.AG_K_CSR_NARROW),
    "fused_dense_bf16x3": (ag.AG_COMPOSE_FUSED, ag.AG_K_BLOCK_DENSE_BF16X3, ag.AG_K_CSR_NARROW),
    "fused_narrow": (ag.AG_COMPOSE_FUSED, ag.AG_K_BLOCK_SPARSE, ag.AG_K_CSR_NARROW),
    "split_sparse_coo": (ag.AG_COMPOSE_SPLIT, ag.AG_K_BLOCK_SPARSE, ag.AG_K_COO),
}
# combinations whose summation order is fixed (no atomics): bitwise reproducible run to run
DETERMINISTIC = [k for k in COMBOS if not k.endswith("coo")]


def usable(name, g, factored=False):
    """The bf16x3 dense kernel exists for unit-weight and for factored matrices only."""
    return not (name.endswith("bf16x3") and g.vals is not None and not factored)


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def force(plan, combo, direction):
    compose, dense, rem = COMBOS[combo]
    ag.ag_plan_force_kernels(plan, ag.AG_CLS_COMPOSE, direction, compose)
    ag.ag_plan_force_kernels(plan, ag.AG_CLS_BLOCKS_DENSE, direction, dense)
    ag.ag_plan_force_kernels(plan, ag.AG_CLS_BLOCKS_SPARSE, direction, ag.AG_K_BLOCK_SPARSE)
    ag.ag_plan_force_kernels(plan, ag.AG_CLS_REMAINDER, direction, rem)


def check(y_gpu, y_ref, S, what):
    y = y_gpu.detach().cpu().numpy().astype(np.float64)
    err = np.abs(y - y_ref)
    bound = REL * S + ABS
    worst = float((err / bound).max()) if err.size else 0.0
    assert np.isfinite(y).all(), f"{what}: non-finite output"
    assert worst <= 1.0, f"{what}: error {worst:.3g} x the bound (max abs err {err.max():.3g})"
    return worst


class Case:
    """One graph + features on the GPU, with oracle results computed once."""

    def __init__(self, g, F, seed=0, layout=ag.AG_LAYOUT_ORIGINAL, factored=False, **opts):
        import torch
        from ag_inputs import features
        self.torch = torch
        self.g, self.F, self.layout, self.factored = g, F, layout, factored
        if factored:                                     # the generator's own factors of the values
            opts = dict(opts, row_scale=g.meta.get("row_scale"), col_scale=g.meta.get("col_scale"))
        self.H = features(g.n, F, 100 + seed)
        self.G = features(g.n, F, 200 + seed)
        self.plan = ag.ag_plan_create(g.rowptr, g.colidx, g.vals, g.n, F, layout=layout, **opts)
        self.exp = ag.ag_plan_export(self.plan)
        self.Yref, self.Sy = oracle.spmm(g.rowptr, g.colidx, g.vals, self.H)
        self.Dref, self.Sd = oracle.spmm_t(g.rowptr, g.colidx, g.vals, self.G)
        self.dev = torch.device("cuda:0")

    def _run(self, fn, X):
        torch = self.torch
        x = torch.from_numpy(X).to(self.dev)
        y = torch.full_like(x, float("nan"))             # stale output must be fully overwritten
        if self.layout == ag.AG_LAYOUT_REORDERED:
            xp = torch.empty_like(x)
            ag.ag_permute_rows(self.plan, x, xp, self.F, False)
            yp = torch.full_like(x, float("nan"))
            fn(self.plan, xp, yp)
            ag.ag_permute_rows(self.plan, yp, y, self.F, True)
        else:
            fn(self.plan, x, y)
        torch.cuda.synchronize()
        return y

    def forward(self):
        return self._run(ag.ag_aggregate, self.H)

    def backward(self):
        return self._run(ag.ag_aggregate_t, self.G)

    def check_all_combos(self, combos=None, directions=(0, 1)):
        out = {}
        for name in (combos or COMBOS):
            if not usable(name, self.g, self.factored):
                continue
            for d in directions:
                say(f"  combo {name} dir {d} n={self.g.n} F={self.F}")
                force(self.plan, name, d)
                if d == 0:
                    out[(name, d)] = check(self.forward(), self.Yref, self.Sy, f"{name} fwd")
                else:
                    out[(name, d)] = check(self.backward(), self.Dref, self.Sd, f"{name} bwd")
        return out

    def close(self):
        ag.ag_plan_destroy(self.plan)
