"""Pins for the oracle's community reordering and intra/inter decomposition.

Expected values are hand-traced from the algorithm statement (comments give
the trace), closed forms (disjoint cliques, edgeless graph) or invariants.
"""
import numpy as np
import pytest

import oracle
from ag_inputs import from_edges, planted_partition, gcn_normalise, directed_random, features
from helpers import dense_from_csr


def ro(g, **kw):
    return oracle.reorder(g.rowptr, g.colidx, **kw)


def test_two_triangles_trace():
    # sweep 0 (threshold 1): 0 joins label 1 (tie 1 vs 2 -> smallest), 1 stays (tie with own),
    # 2 joins label 1 (weight 2); same for 3,4,5 -> label 4.  Sweep 1 moves nothing.
    # coarse level: two isolated nodes, nothing merges.
    g = from_edges(6, [0, 0, 1, 3, 3, 4], [1, 2, 2, 4, 5, 5])
    r = ro(g, block_cap=128, min_block=1)
    assert r.comm.tolist() == [0, 0, 0, 1, 1, 1]
    assert r.blk_ptr.tolist() == [0, 3, 6]
    assert r.perm.tolist() == [0, 1, 2, 3, 4, 5]


def test_path_of_four_trace_no_cap():
    # sweep 0: 0->label1, 1 stays, 2->label1 (tie 1 vs 3 -> smallest), 3->label1. sweep 1: stable.
    g = from_edges(4, [0, 1, 2], [1, 2, 3])
    r = ro(g, block_cap=128, min_block=1)
    assert r.comm.tolist() == [0, 0, 0, 0]
    assert r.blk_ptr.tolist() == [0, 4]


def test_path_of_four_trace_cap_two():
    # cap 2.  sweep 0: 0->label1 (size 2); 1 stays; 2: label1 is full -> joins label3; 3 stays.
    # sweep 1 (threshold 2 for inner nodes): 1 is weakly attached (1 < 2) but its own label is
    # the current one and no neighbour label reaches 2 -> stays; 2 is weakly attached to label3,
    # its home label 2 is empty -> goes home; 3 (total weight 1, threshold 1) follows to label2.
    # sweep 2: stable.  clusters {0,1},{2,3}; coarse level cannot merge (2+2 > cap).
    g = from_edges(4, [0, 1, 2], [1, 2, 3])
    r = ro(g, block_cap=2, min_block=2)
    assert r.comm.tolist() == [0, 0, 1, 1]
    assert r.blk_ptr.tolist() == [0, 2, 4]
    assert r.perm.tolist() == [0, 1, 2, 3]


def test_star_trace():
    # centre 0 joins label 1 (smallest of equal candidates); every leaf then joins label 1.
    g = from_edges(5, [0, 0, 0, 0], [1, 2, 3, 4])
    r = ro(g, block_cap=128, min_block=1)
    assert r.comm.tolist() == [0] * 5


def test_layout_blocks_then_tail_trace():
    # triangle {1,3,5}, edge {0,4}, isolated 2.  min_block 3 -> only the triangle is a block.
    # community ids by smallest member: {0,4}->0, {1,3,5}->1, {2}->2.
    g = from_edges(6, [1, 1, 3, 0], [3, 5, 5, 4])
    r = ro(g, block_cap=128, min_block=3)
    assert r.comm.tolist() == [0, 1, 2, 1, 0, 1]
    assert r.blk_ptr.tolist() == [0, 3]
    assert r.perm.tolist() == [1, 3, 5, 0, 2, 4]
    assert r.iperm.tolist() == [3, 0, 4, 1, 5, 2]


def test_edgeless_graph_identity_no_blocks():
    g = from_edges(10, np.empty(0, int), np.empty(0, int))
    r = ro(g)
    assert r.perm.tolist() == list(range(10))
    assert r.blk_ptr.tolist() == [0]


def test_disjoint_cliques_become_blocks_exactly():
    rng = np.random.default_rng(5)
    sizes = [16, 40, 128, 23, 64]
    n = sum(sizes) + 7                      # 7 isolated vertices
    ids = rng.permutation(n)
    us, vs, at = [], [], 0
    members = []
    for s in sizes:
        m = ids[at:at + s]
        members.append(set(m.tolist()))
        iu, ju = np.triu_indices(s, 1)
        us.append(m[iu]); vs.append(m[ju])
        at += s
    g = from_edges(n, np.concatenate(us), np.concatenate(vs))
    r = ro(g, block_cap=128, min_block=16)
    assert r.blk_ptr.size - 1 == len(sizes)
    got = [set(r.perm[r.blk_ptr[b]:r.blk_ptr[b + 1]].tolist()) for b in range(len(sizes))]
    assert sorted(map(sorted, got)) == sorted(map(sorted, members))
    # blocks ordered by smallest member, members ascending, tail ascending
    mins = [min(s) for s in got]
    assert mins == sorted(mins)
    for b in range(len(sizes)):
        blk = r.perm[r.blk_ptr[b]:r.blk_ptr[b + 1]]
        assert np.all(np.diff(blk) > 0)
    tail = r.perm[r.blk_ptr[-1]:]
    assert tail.size == 7 and np.all(np.diff(tail) > 0)
    s = oracle.split(g.rowptr, g.colidx, None, r.perm, r.iperm, r.blk_ptr)
    # density 1 in every block; the remainder holds only the tail's self loops
    assert int(s.intra_rowptr[-1]) == sum(x * x for x in sizes)
    assert int(s.inter_rowptr[-1]) == 7


@pytest.mark.parametrize("seed", [1, 2])
def test_invariants_on_sbm(seed):
    g = planted_partition(24, 64, 8, 0.8, seed)
    r = ro(g, block_cap=64, min_block=16)
    n = g.n
    assert sorted(r.perm.tolist()) == list(range(n))
    assert np.array_equal(r.iperm[r.perm], np.arange(n))
    sizes = np.diff(r.blk_ptr)
    assert sizes.min() >= 16 and sizes.max() <= 64
    csize = np.bincount(r.comm)
    tail = r.perm[r.blk_ptr[-1]:]
    assert np.all(csize[r.comm[tail]] < 16)
    assert np.all(np.diff(tail) > 0)
    # every block is one community
    for b in range(sizes.size):
        assert np.unique(r.comm[r.perm[r.blk_ptr[b]:r.blk_ptr[b + 1]]]).size == 1
    # the reordering recovers most planted structure
    s = oracle.split(g.rowptr, g.colidx, None, r.perm, r.iperm, r.blk_ptr)
    frac = (int(s.intra_rowptr[-1]) - int(r.blk_ptr[-1])) / (g.nnz - n)
    assert frac > 0.6, frac


def test_direction_of_edges_does_not_matter():
    g = directed_random(300, 2.0, 3, weighted=False)
    # same pattern with every arc reversed
    rows = np.repeat(np.arange(g.n), np.diff(g.rowptr))
    from ag_inputs.graphs import _csr_from_directed
    gt = _csr_from_directed(g.n, g.colidx.astype(np.int64), rows.astype(np.int64))
    a, b = ro(g, min_block=4), ro(gt, min_block=4)
    assert np.array_equal(a.perm, b.perm) and np.array_equal(a.blk_ptr, b.blk_ptr)


def test_split_partitions_entries_and_keeps_values():
    g = gcn_normalise(planted_partition(10, 32, 6, 0.75, 4))
    r = ro(g, block_cap=32, min_block=8)
    s = oracle.split(g.rowptr, g.colidx, g.vals, r.perm, r.iperm, r.blk_ptr)
    n = g.n
    A = dense_from_csr(g.rowptr, g.colidx, g.vals)
    PA = A[np.ix_(r.perm, r.perm)]                      # P A P^T
    Ai = dense_from_csr(s.intra_rowptr, s.intra_col, s.intra_val)
    Ao = dense_from_csr(s.inter_rowptr, s.inter_col, s.inter_val)
    assert np.array_equal(Ai + Ao, PA)                  # values carried bit-exactly
    assert not np.any((Ai != 0) & (Ao != 0))            # disjoint
    assert int(s.intra_rowptr[-1]) + int(s.inter_rowptr[-1]) == g.nnz
    blk = np.full(n, -1)
    for b in range(r.blk_ptr.size - 1):
        blk[r.blk_ptr[b]:r.blk_ptr[b + 1]] = b
    ri, ci = np.nonzero(Ai)
    assert np.all((blk[ri] == blk[ci]) & (blk[ri] >= 0))
    ro_, co = np.nonzero(Ao)
    assert np.all((blk[ro_] != blk[co]) | (blk[ro_] < 0))
    for rp, c in ((s.intra_rowptr, s.intra_col), (s.inter_rowptr, s.inter_col)):
        for i in range(n):
            assert np.all(np.diff(c[rp[i]:rp[i + 1]]) > 0)
    assert sorted(np.concatenate([s.intra_val, s.inter_val]).tolist()) == sorted(g.vals.tolist())


def test_permutation_invariance_of_aggregation():
    g = gcn_normalise(planted_partition(12, 32, 6, 0.7, 6))
    r = ro(g, block_cap=32, min_block=8)
    s = oracle.split(g.rowptr, g.colidx, g.vals, r.perm, r.iperm, r.blk_ptr)
    H = features(g.n, 6, 2)
    Y = oracle.spmm(g.rowptr, g.colidx, g.vals, H, want_abs=False)
    Hp = H[r.perm]
    Yp = (oracle.spmm(s.intra_rowptr, s.intra_col, s.intra_val, Hp, want_abs=False)
          + oracle.spmm(s.inter_rowptr, s.inter_col, s.inter_val, Hp, want_abs=False))
    np.testing.assert_allclose(Yp[r.iperm], Y, rtol=1e-12, atol=1e-14)


def test_golden_trace_fixture():
    # every hand-traced case of tests/golden/reorder_traces.txt (the traces are written out there)
    from helpers import failing_reorder_traces, reorder_trace_cases
    assert len(reorder_trace_cases()) >= 27
    assert failing_reorder_traces(oracle.reorder) == []


def test_ordering_levels_put_connected_communities_next_to_each_other():
    # 12 cliques of 16; cliques (2k, 2k+1) are joined by 6 edges, nothing else.  With ids shuffled
    # the flat order (by smallest member) interleaves the pairs; the ordering levels must make
    # every pair adjacent.  Each clique stays its own block (cap 16).
    rng = np.random.default_rng(3)
    n, s = 12 * 16, 16
    ids = rng.permutation(n)
    us, vs = [], []
    groups = [ids[k * s:(k + 1) * s] for k in range(12)]
    for m in groups:
        iu, ju = np.triu_indices(s, 1)
        us.append(m[iu]); vs.append(m[ju])
    for k in range(0, 12, 2):
        us.append(groups[k][:6]); vs.append(groups[k + 1][:6])
    g = from_edges(n, np.concatenate(us), np.concatenate(vs))
    pair_of = np.empty(n, int)
    for k, m in enumerate(groups):
        pair_of[m] = k // 2
    flat = ro(g, block_cap=16, min_block=16, order_levels=0)
    hier = ro(g, block_cap=16, min_block=16, order_levels=3)
    assert flat.blk_ptr.tolist() == hier.blk_ptr.tolist() == list(range(0, n + 1, 16))
    assert sorted(hier.perm.tolist()) == list(range(n))
    def block_pairs(r):
        return [int(pair_of[r.perm[b * 16]]) for b in range(12)]
    hp = block_pairs(hier)
    assert all(hp[2 * i] == hp[2 * i + 1] for i in range(6)), hp        # partners are adjacent
    fp = block_pairs(flat)
    assert any(fp[2 * i] != fp[2 * i + 1] for i in range(6)), fp        # (they were not before)
    # same communities either way
    assert np.array_equal(np.sort(flat.comm), np.sort(hier.comm))
