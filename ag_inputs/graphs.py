"""Seeded synthetic graph / feature generators (numpy, PCG64).

Everything here is input preparation only.  A graph is handed out as a CSR
matrix whose rows are destination vertices and whose column indices are source
vertices, optionally with fp32 edge values (None = unit weights).

The recipes stand in for the public GNN datasets the paper evaluates on (its
dataset table): community-clustered graphs whose vertex numbering is random,
power-law degree graphs, and a graph that mixes a dense-community half with a
uniformly sparse half.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Optional

import numpy as np

__all__ = [
    "Graph", "planted_partition", "chung_lu_communities", "mixed_density",
    "directed_random", "from_edges", "gcn_normalise", "row_normalise",
    "features", "glorot_uniform", "labels", "config_graph", "CONFIGS",
]


@dataclass
class Graph:
    n: int
    rowptr: np.ndarray            # int32 [n+1]
    colidx: np.ndarray            # int32 [nnz], ascending inside each row
    vals: Optional[np.ndarray]    # float32 [nnz] or None (unit weights)
    meta: dict = field(default_factory=dict)

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])

    def degrees(self) -> np.ndarray:
        return np.diff(self.rowptr)


def _rng(seed: int) -> np.random.Generator:
    return np.random.default_rng(np.random.PCG64(seed))


# --------------------------------------------------------------------------- #
# CSR assembly
# --------------------------------------------------------------------------- #
def _csr_from_directed(n: int, rows: np.ndarray, cols: np.ndarray,
                       vals: Optional[np.ndarray] = None) -> Graph:
    """Sort (row, col) pairs, drop exact duplicates, build CSR."""
    key = rows.astype(np.int64) * n + cols.astype(np.int64)
    if vals is None:
        key = np.unique(key)
        v = None
    else:
        key, first = np.unique(key, return_index=True)
        v = np.ascontiguousarray(vals[first], dtype=np.float32)
    r = (key // n).astype(np.int64)
    c = (key % n).astype(np.int32)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.bincount(r, minlength=n), out=rowptr[1:])
    assert rowptr[-1] < 2 ** 31
    return Graph(n, rowptr.astype(np.int32), np.ascontiguousarray(c), v)


def from_edges(n: int, u: np.ndarray, v: np.ndarray, *, self_loops: bool = True,
               symmetric: bool = True) -> Graph:
    """CSR pattern from an edge list; `symmetric` stores both directions."""
    u = np.asarray(u, dtype=np.int64)
    v = np.asarray(v, dtype=np.int64)
    rows = [u]
    cols = [v]
    if symmetric:
        rows.append(v)
        cols.append(u)
    if self_loops:
        d = np.arange(n, dtype=np.int64)
        rows.append(d)
        cols.append(d)
    return _csr_from_directed(n, np.concatenate(rows), np.concatenate(cols))


def gcn_normalise(g: Graph) -> Graph:
    """Attach values D^-1/2 (A+I) D^-1/2 (computed in fp64, rounded to fp32).

    The pattern is expected to already contain the self-loops; the degree is
    the row's stored entry count.
    """
    deg = np.diff(g.rowptr).astype(np.float64)
    deg[deg == 0] = 1.0
    inv = 1.0 / np.sqrt(deg)
    rows = np.repeat(np.arange(g.n, dtype=np.int64), np.diff(g.rowptr))
    vals = (inv[rows] * inv[g.colidx]).astype(np.float32)
    scale = inv.astype(np.float32)                       # vals[i][j] ~ scale[i] * scale[j]
    return Graph(g.n, g.rowptr, g.colidx, vals, dict(g.meta, norm="gcn", row_scale=scale, col_scale=scale))


def row_normalise(g: Graph) -> Graph:
    """Attach values D^-1 (A+I): the mean aggregator; NOT symmetric."""
    deg = np.diff(g.rowptr).astype(np.float64)
    deg[deg == 0] = 1.0
    rows = np.repeat(np.arange(g.n, dtype=np.int64), np.diff(g.rowptr))
    vals = (1.0 / deg[rows]).astype(np.float32)
    return Graph(g.n, g.rowptr, g.colidx, vals, dict(g.meta, norm="row", row_scale=(1.0 / deg).astype(np.float32),
                                                     col_scale=None))


# --------------------------------------------------------------------------- #
# de-duplicated pair sampling
# --------------------------------------------------------------------------- #
def _unique_pairs(n: int, need: int, draw: Callable[[int], tuple],
                  exclude: Optional[np.ndarray] = None, oversample: float = 1.15,
                  max_rounds: int = 400) -> np.ndarray:
    """Draw unordered pairs until exactly `need` distinct ones were seen.

    Returns int64 keys lo*n+hi in order of first arrival.  `exclude` holds keys
    that must not be produced again (sorted int64).
    """
    kept = np.empty(0, dtype=np.int64)
    for _ in range(max_rounds):
        missing = need - kept.size
        if missing <= 0:
            break
        a, b = draw(int(missing * oversample) + 64)
        lo = np.minimum(a, b).astype(np.int64)
        hi = np.maximum(a, b).astype(np.int64)
        ok = lo != hi
        key = lo[ok] * n + hi[ok]
        if exclude is not None and exclude.size:
            pos = np.searchsorted(exclude, key)
            pos[pos >= exclude.size] = exclude.size - 1
            key = key[exclude[pos] != key]
        allk = np.concatenate([kept, key])
        _, first = np.unique(allk, return_index=True)
        first.sort()
        kept = allk[first][:need]
    if kept.size != need:
        raise RuntimeError(f"could not draw {need} distinct pairs (got {kept.size})")
    return kept


def _finish(n: int, keys: np.ndarray, comm: np.ndarray, rng: np.random.Generator,
            *, shuffle: bool, self_loops: bool = True) -> Graph:
    u = keys // n
    v = keys % n
    if shuffle:
        p = rng.permutation(n).astype(np.int64)   # new id of old vertex x is p[x]
        u, v = p[u], p[v]
        comm_new = np.empty_like(comm)
        comm_new[p] = comm
        comm = comm_new
    g = from_edges(n, u, v, self_loops=self_loops, symmetric=True)
    cu, cv = comm[u], comm[v]
    intra = int(np.count_nonzero((cu == cv) & (cu >= 0)))
    g.meta.update(
        planted=comm.astype(np.int32), edges=int(keys.size),
        planted_intra_frac=intra / max(1, keys.size),
        avg_degree=2.0 * keys.size / n, max_degree=int(np.diff(g.rowptr).max()),
    )
    return g


# --------------------------------------------------------------------------- #
# recipes
# --------------------------------------------------------------------------- #
def planted_partition(n_comm: int, comm_size: int, avg_degree: float,
                      intra_frac: float, seed: int, *, shuffle: bool = True) -> Graph:
    """Stochastic-block-model style graph with exact edge counts.

    M = n*avg_degree/2 undirected edges; round(M*intra_frac) of them join two
    distinct members of one uniformly chosen community, the rest join vertices
    of different communities, all de-duplicated.
    """
    rng = _rng(seed)
    n = n_comm * comm_size
    m = int(round(n * avg_degree / 2))
    m_in = int(round(m * intra_frac))
    m_out = m - m_in
    comm = np.repeat(np.arange(n_comm, dtype=np.int64), comm_size)

    def draw_in(k):
        c = rng.integers(0, n_comm, size=k, dtype=np.int64) * comm_size
        return (c + rng.integers(0, comm_size, size=k, dtype=np.int64),
                c + rng.integers(0, comm_size, size=k, dtype=np.int64))

    def draw_out(k):
        a = rng.integers(0, n, size=k, dtype=np.int64)
        b = rng.integers(0, n, size=k, dtype=np.int64)
        ok = (a // comm_size) != (b // comm_size)
        return a[ok], b[ok]

    k_in = _unique_pairs(n, m_in, draw_in)
    k_out = _unique_pairs(n, m_out, draw_out) if m_out else np.empty(0, np.int64)
    g = _finish(n, np.concatenate([k_in, k_out]), comm, rng, shuffle=shuffle)
    g.meta.update(kind="planted_partition", n_comm=n_comm, comm_size=comm_size)
    return g


def _powerlaw_weights(n: int, exponent: float, w_max: float, w_mean: float) -> np.ndarray:
    """w_r = c (r + r0)^(-1/(exponent-1)), r = 0..n-1, with max and mean fixed."""
    g = 1.0 / (exponent - 1.0)
    r = np.arange(n, dtype=np.float64)

    def mean_for(r0):
        c = w_max * r0 ** g
        return c * np.mean((r + r0) ** (-g))

    lo, hi = 1e-9, 1e9
    for _ in range(200):              # mean_for is increasing in r0
        mid = np.sqrt(lo * hi)
        if mean_for(mid) < w_mean:
            lo = mid
        else:
            hi = mid
    r0 = np.sqrt(lo * hi)
    return w_max * r0 ** g * (r + r0) ** (-g)


def chung_lu_communities(n: int, exponent: float, avg_degree: float, max_degree: float,
                         intra_frac: float, comm_lo: int, comm_hi: int, seed: int,
                         *, shuffle: bool = True) -> Graph:
    """Chung-Lu style power-law graph with planted communities of random size."""
    rng = _rng(seed)
    w = _powerlaw_weights(n, exponent, max_degree, avg_degree)
    w = w[rng.permutation(n)]
    sizes = []
    left = n
    while left > 0:
        s = int(rng.integers(comm_lo, comm_hi + 1))
        if s >= left:
            s = left
        elif left - s < comm_lo:
            s = left
        sizes.append(s)
        left -= s
    sizes = np.asarray(sizes, dtype=np.int64)
    cstart = np.concatenate([[0], np.cumsum(sizes)])
    comm = np.repeat(np.arange(sizes.size, dtype=np.int64), sizes)
    cum0 = np.concatenate([[0.0], np.cumsum(w)])
    total = cum0[-1]
    m = int(round(n * avg_degree / 2))
    m_in = int(round(m * intra_frac))
    m_out = m - m_in

    def pick(k):
        x = rng.random(k) * total
        return np.clip(np.searchsorted(cum0, x, side="right") - 1, 0, n - 1)

    def draw_in(k):
        a = pick(k)
        lo = cstart[comm[a]]
        hi = cstart[comm[a] + 1]
        x = cum0[lo] + rng.random(k) * (cum0[hi] - cum0[lo])
        b = np.clip(np.searchsorted(cum0, x, side="right") - 1, lo, hi - 1)
        return a, b

    def draw_out(k):
        a, b = pick(k), pick(k)
        ok = comm[a] != comm[b]
        return a[ok], b[ok]

    k_in = _unique_pairs(n, m_in, draw_in, oversample=2.0)
    k_out = _unique_pairs(n, m_out, draw_out, oversample=1.3)
    g = _finish(n, np.concatenate([k_in, k_out]), comm, rng, shuffle=shuffle)
    g.meta.update(kind="chung_lu", n_comm=int(sizes.size))
    return g


def mixed_density(n_comm: int, comm_size: int, p_dense: float, sparse_degree: float,
                  cross_frac: float, seed: int, *, shuffle: bool = True) -> Graph:
    """Half the vertices in dense communities, half uniformly sparse, plus cross edges."""
    rng = _rng(seed)
    nd = n_comm * comm_size
    n = 2 * nd
    iu, ju = np.triu_indices(comm_size, k=1)
    iu = iu.astype(np.int64)
    ju = ju.astype(np.int64)
    keys = []
    chunk = max(1, (1 << 24) // iu.size)
    for c0 in range(0, n_comm, chunk):
        c1 = min(n_comm, c0 + chunk)
        mask = rng.random((c1 - c0, iu.size), dtype=np.float32) < np.float32(p_dense)
        cc, pp = np.nonzero(mask)
        base = (cc.astype(np.int64) + c0) * comm_size
        keys.append((base + iu[pp]) * n + (base + ju[pp]))
    k_dense = np.concatenate(keys)
    m_sparse = int(round(nd * sparse_degree / 2))

    def draw_sparse(k):
        return (nd + rng.integers(0, nd, size=k, dtype=np.int64),
                nd + rng.integers(0, nd, size=k, dtype=np.int64))

    k_sparse = _unique_pairs(n, m_sparse, draw_sparse)
    have = np.sort(np.concatenate([k_dense, k_sparse]))
    m_cross = int(round(cross_frac * have.size))

    def draw_cross(k):
        return (rng.integers(0, n, size=k, dtype=np.int64),
                rng.integers(0, n, size=k, dtype=np.int64))

    k_cross = _unique_pairs(n, m_cross, draw_cross, exclude=have) if m_cross else np.empty(0, np.int64)
    comm = np.concatenate([np.repeat(np.arange(n_comm, dtype=np.int64), comm_size),
                           np.full(nd, -1, dtype=np.int64)])
    g = _finish(n, np.concatenate([k_dense, k_sparse, k_cross]), comm, rng, shuffle=shuffle)
    g.meta.update(kind="mixed_density", n_comm=n_comm, comm_size=comm_size)
    return g


def rmat(n: int, n_edges: int, seed: int, *, a: float = 0.57, b: float = 0.19, c: float = 0.19,
         self_loops: bool = True) -> Graph:
    """Undirected R-MAT graph (recursive-matrix generator: every edge picks one quadrant of the
    adjacency matrix per bit level with probabilities a, b, c, 1-a-b-c) on n vertices, the kind of
    synthetic graph the paper sweeps over densities in Sec. 2.1.  Ids are drawn on the next power
    of two and pairs that fall outside [0, n), loops and duplicates are drawn again until exactly
    n_edges distinct undirected edges exist."""
    rng = _rng(seed)
    bits = max(1, int(np.ceil(np.log2(max(2, n)))))
    n_edges = int(min(n_edges, n * (n - 1) // 2))

    def draw(k):
        u = np.zeros(k, dtype=np.int64)
        v = np.zeros(k, dtype=np.int64)
        for _ in range(bits):
            x = rng.random(k)
            right = ((x >= a) & (x < a + b)) | (x >= a + b + c)      # quadrants b and d: column bit set
            down = x >= a + b                                        # quadrants c and d: row bit set
            u = (u << 1) | down
            v = (v << 1) | right
        ok = (u < n) & (v < n)
        return u[ok], v[ok]

    keys = _unique_pairs(n, n_edges, draw, oversample=1.5) if n_edges else np.empty(0, np.int64)
    g = _finish(n, keys, np.full(n, -1, dtype=np.int64), rng, shuffle=True, self_loops=self_loops)
    g.meta.update(kind="rmat", a=a, b=b, c=c)
    return g


def directed_random(n: int, avg_out_degree: float, seed: int, *, self_loops: bool = True,
                    weighted: bool = True) -> Graph:
    """Uniform random *directed* graph (non-symmetric pattern and values)."""
    rng = _rng(seed)
    m = int(round(n * avg_out_degree))
    r = rng.integers(0, n, size=m, dtype=np.int64)
    c = rng.integers(0, n, size=m, dtype=np.int64)
    if self_loops:
        d = np.arange(n, dtype=np.int64)
        r = np.concatenate([r, d])
        c = np.concatenate([c, d])
    g = _csr_from_directed(n, r, c)
    if weighted:
        g.vals = rng.uniform(-1.0, 1.0, size=g.nnz).astype(np.float32)
    g.meta.update(kind="directed_random")
    return g


# --------------------------------------------------------------------------- #
# dense inputs
# --------------------------------------------------------------------------- #
def features(n: int, f: int, seed: int) -> np.ndarray:
    """fp32 N(0,1) matrix, row-major n x f."""
    return _rng(seed).standard_normal((n, f), dtype=np.float32)


def glorot_uniform(fan_in: int, fan_out: int, seed: int) -> np.ndarray:
    a = np.sqrt(6.0 / (fan_in + fan_out))
    return _rng(seed).uniform(-a, a, size=(fan_in, fan_out)).astype(np.float32)


def labels(n: int, n_class: int, seed: int) -> np.ndarray:
    return _rng(seed).integers(0, n_class, size=n, dtype=np.int32)


# --------------------------------------------------------------------------- #
# the five benchmark workloads (index = position in the configs list, 0-based)
# --------------------------------------------------------------------------- #
CONFIGS = [
    dict(name="sbm4k", kind="sbm", n_comm=64, comm_size=64, deg=8, intra=0.80, F=16, norm="gcn"),
    dict(name="sbm64k", kind="sbm", n_comm=512, comm_size=128, deg=16, intra=0.70, F=64, norm="gcn"),
    dict(name="chunglu256k", kind="cl", n=262144, exponent=2.1, deg=50, max_deg=20000, intra=0.60,
         comm_lo=32, comm_hi=1024, F=128, norm="gcn"),
    dict(name="sbm1m_gcn", kind="sbm", n_comm=8192, comm_size=128, deg=20, intra=0.65, F=128,
         hidden=256, classes=16, norm="gcn"),
    dict(name="mixed1m_gin", kind="mixed", n_comm=4096, comm_size=128, p=0.3, sparse_deg=6,
         cross=0.02, F=32, norm="unit"),
]


def config_graph(index: int, *, scale: float = 1.0) -> Graph:
    """Graph of benchmark workload `index` (seed 1000+index).

    `scale` < 1 shrinks the vertex count (number of communities) for tests while
    keeping community size, degree and mixing.
    """
    c = CONFIGS[index]
    seed = 1000 + index
    if c["kind"] == "sbm":
        g = planted_partition(max(2, int(round(c["n_comm"] * scale))), c["comm_size"], c["deg"],
                              c["intra"], seed)
    elif c["kind"] == "cl":
        n = max(4096, int(round(c["n"] * scale)))
        g = chung_lu_communities(n, c["exponent"], c["deg"], min(c["max_deg"], n // 8),
                                 c["intra"], c["comm_lo"], c["comm_hi"], seed)
    else:
        g = mixed_density(max(2, int(round(c["n_comm"] * scale))), c["comm_size"], c["p"],
                          c["sparse_deg"], c["cross"], seed)
    if c["norm"] == "gcn":
        g = gcn_normalise(g)
    g.meta.update(config=index, name=c["name"], F=c["F"])
    return g
