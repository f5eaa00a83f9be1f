"""The synthetic inputs have the structure the benchmark configs ask for."""
import numpy as np

from ag_inputs import config_graph, planted_partition, chung_lu_communities, mixed_density


def _symmetric(g):
    rows = np.repeat(np.arange(g.n, dtype=np.int64), np.diff(g.rowptr))
    k1 = np.sort(rows * g.n + g.colidx)
    k2 = np.sort(g.colidx.astype(np.int64) * g.n + rows)
    return np.array_equal(k1, k2)


def test_config0_exact_counts():
    g = config_graph(0)
    assert g.n == 4096 and g.nnz == 36864
    assert abs(g.meta["planted_intra_frac"] - 0.8) < 1e-3
    assert _symmetric(g)
    rows = np.repeat(np.arange(g.n), np.diff(g.rowptr))
    assert np.count_nonzero(rows == g.colidx) == g.n        # self loops
    deg = np.diff(g.rowptr).astype(np.float64)
    np.testing.assert_allclose(g.vals, (1 / np.sqrt(deg[rows] * deg[g.colidx])).astype(np.float32))
    # deterministic under the seed
    g2 = config_graph(0)
    assert np.array_equal(g.colidx, g2.colidx) and np.array_equal(g.vals, g2.vals)


def test_config1_exact_counts():
    g = config_graph(1)
    assert g.n == 65536 and g.nnz == 1114112
    assert abs(g.meta["planted_intra_frac"] - 0.7) < 1e-3


def test_scaled_shapes_of_other_configs():
    g = config_graph(2, scale=1 / 16)
    assert abs(g.meta["avg_degree"] - 50) < 1 and abs(g.meta["planted_intra_frac"] - 0.6) < 0.01
    assert g.meta["max_degree"] > 500                      # hubs exist
    g = config_graph(4, scale=1 / 64)
    assert g.vals is None and abs(g.meta["avg_degree"] - 22.5) < 0.5
    assert _symmetric(g)
    g = config_graph(3, scale=1 / 64)
    assert abs(g.meta["avg_degree"] - 20) < 1e-6 and abs(g.meta["planted_intra_frac"] - 0.65) < 1e-3


def test_ids_are_shuffled():
    g = planted_partition(16, 32, 6, 0.8, 1)
    p = g.meta["planted"]
    assert np.count_nonzero(np.diff(p) != 0) > g.n // 2     # neighbours in id are rarely co-members


def test_rmat_graph_has_exact_edge_count_and_a_skewed_degree_distribution():
    from ag_inputs import rmat
    import numpy as np
    n, m = 19717, 60000
    g = rmat(n, m, 7)
    assert g.n == n and g.nnz == 2 * m + n                      # both directions + the diagonal
    rows = np.repeat(np.arange(n), np.diff(g.rowptr))
    key = rows.astype(np.int64) * n + g.colidx
    assert np.array_equal(np.sort(key), np.sort(g.colidx.astype(np.int64) * n + rows))   # symmetric pattern
    deg = np.diff(g.rowptr) - 1
    assert deg.max() > 20 * deg.mean()                          # hubs, unlike a uniform random graph
    g2 = rmat(n, m, 7)
    assert np.array_equal(g.colidx, g2.colidx)                  # seeded
