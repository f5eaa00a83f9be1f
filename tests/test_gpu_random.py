"""GPU parity on seeded random matrices: random size, density, symmetry, weights, feature width
and decomposition options, every kernel combination, forward and backward."""
import numpy as np
import pytest

import paper_2305_17408_amd as ag
from ag_inputs.graphs import _csr_from_directed
from gpu_util import Case, say

pytestmark = pytest.mark.gpu


def random_case(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 3000))
    deg = float(rng.choice([0.5, 2, 8, 30]))
    m = int(n * deg)
    k = int(rng.integers(1, max(2, n // 40) + 1))
    grp = rng.integers(0, k, size=n)
    order = np.argsort(grp, kind="stable")
    start = np.searchsorted(grp[order], np.arange(k + 1))
    r = rng.integers(0, n, size=m)
    intra = rng.random(m) < rng.choice([0.0, 0.5, 0.9])
    c = rng.integers(0, n, size=m)
    gi = grp[r]
    lo, hi = start[gi], start[gi + 1]
    c_in = order[np.minimum(lo + (rng.random(m) * np.maximum(hi - lo, 1)).astype(np.int64), n - 1)]
    c = np.where(intra, c_in, c)
    if rng.random() < 0.6:
        r, c = np.concatenate([r, c]), np.concatenate([c, r])
    if rng.random() < 0.7:
        d = np.arange(n)
        r, c = np.concatenate([r, d]), np.concatenate([c, d])
    g = _csr_from_directed(n, r.astype(np.int64), c.astype(np.int64))
    if rng.random() < 0.7 and g.nnz:
        g.vals = rng.uniform(-1.5, 1.5, size=g.nnz).astype(np.float32)
    F = int(rng.choice([1, 2, 4, 8, 12, 16, 31, 32, 64, 100, 128, 160]))
    opts = dict(block_cap=int(rng.choice([16, 32, 64, 100, 128, 200, 256])), min_block=int(rng.choice([1, 4, 16])),
                dense_density=float(rng.choice([0.05, 0.2])))
    layout = int(rng.integers(0, 2))
    return g, F, opts, layout


@pytest.mark.parametrize("seed", range(24))
def test_random_matrix(seed):
    g, F, opts, layout = random_case(1000 + seed)
    say(f"seed {seed}: n={g.n} nnz={g.nnz} F={F} weighted={g.vals is not None} layout={layout} {opts}")
    c = Case(g, F, seed=seed, layout=layout, **opts)
    st = ag.ag_plan_stats(c.plan)
    say(f"   blocks={st['n_blocks']} dense={st['n_dense_blocks']} symmetric={st['symmetric']} long={st['n_long_rows']}")
    c.check_all_combos()
    c.close()
