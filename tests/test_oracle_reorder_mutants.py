"""Do the hand-traced reorder cases really pin the oracle's reordering?

Each case below plants ONE mistake in a scratch copy of oracle/ag_oracle.c (a textual patch of the
rule named in its id), compiles the copy with gcc and runs the hand-traced cases of
tests/golden/reorder_traces.txt against it.  Every planted mistake must make at least one traced
case fail; the unpatched copy must pass them all.  Nothing here touches the HIP library: the
expected values are the hand traces, so a wrong rule in the oracle cannot hide behind a second
implementation that shares it.  CPU only.
"""
import ctypes
import os
import subprocess
from types import SimpleNamespace

import numpy as np
import pytest

from helpers import failing_reorder_traces

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "ag_oracle.c")

CMP_ASC = "i32 x = *(const i32 *)a, y = *(const i32 *)b;\n    return (x > y) - (x < y);"
CMP_DESC = "i32 x = *(const i32 *)a, y = *(const i32 *)b;\n    return (x < y) - (x > y);"

# id -> list of (text in the oracle, replacement); each text must occur exactly once
MUTANTS = {
    # contraction
    "parallel_edges_not_summed": [("c->ew[out - 1] += arcs[p].w;", ";")],
    "node_weights_not_summed": [("c->nw[cluster[v]] += g->nw[v];", "c->nw[cluster[v]] = 1;")],
    "inner_edges_kept": [("if (cu != cv) { arcs[pos[cv]]", "if (1) { arcs[pos[cv]]"),
                         ("if (cluster[g->adj[e]] != cluster[v]) cnt", "if (1) cnt")],
    # joining threshold / weak attachment
    "threshold_always_1": [("i64 thr = ((level == 0 && s == 0) || tot[v] < 2) ? 1 : 2;", "i64 thr = 1;")],
    "threshold_3_instead_of_2": [("|| tot[v] < 2) ? 1 : 2;", "|| tot[v] < 2) ? 1 : 3;")],
    "first_sweep_lenient_on_every_level": [("(level == 0 && s == 0)", "(s == 0)")],
    "no_exception_for_light_nodes": [("|| tot[v] < 2)", ")")],
    "no_return_to_own_label": [("if (size[cur] > g->nw[v] && size[v] == 0) best = v;", ";")],
    # choice among labels
    "ties_to_largest_label": [(CMP_ASC, CMP_DESC)],
    "current_label_not_preferred": [("conn[L] > bw) {", "conn[L] >= bw && conn[L] > 0) {")],
    "cap_off_by_one": [("size[L] + g->nw[v] <= cap", "size[L] + g->nw[v] < cap")],
    "sizes_not_updated_during_sweep": [("size[cur] -= g->nw[v];\n                size[best] += g->nw[v];", ";")],
    # level loop
    "stop_rule_dropped": [("&& ((i64)20 * k <= (i64)19 * g.n)", "")],
    "stop_rule_10_percent": [("(i64)20 * k <= (i64)19 * g.n", "(i64)10 * k <= (i64)9 * g.n")],
    "stop_rule_strict": [("(i64)20 * k <= (i64)19 * g.n", "(i64)20 * k < (i64)19 * g.n")],
    "no_second_level": [("int go_on = (k < g.n)", "int go_on = 0 && (k < g.n)")],
    # ordering levels and layout
    "ordering_keys_reversed": [("ord[c].key[2 - ol] = at_node[c];", "ord[c].key[ol] = at_node[c];")],
    "ordering_cap_not_scaled": [("cap2 *= 8;", "cap2 *= 1;")],
    "ordering_levels_run_as_level_0": [("propagate_level(&cg, 1 + ol,", "propagate_level(&cg, 0,")],
    "min_block_strict": [("if (csize[c] >= min_block)", "if (csize[c] > min_block)")],
    # second method: agglomeration by modularity gain
    "gain_without_degree_term": [("const i64 gain = conn[r] * M2 - deg[u] * deg[r];", "const i64 gain = conn[r] * M2;")],
    "gain_degrees_not_accumulated": [("deg[best] += deg[u];", ";")],
    "gain_sizes_not_accumulated": [("size[best] += size[u];", ";")],
    "gain_zero_accepted": [("if (gain > 0 && size[u] + size[r] <= cap &&", "if (gain >= 0 && size[u] + size[r] <= cap &&"),
                           ("i64 best_gain = 0;\n        for (i32 c = 0; c < nc; ++c) {", "i64 best_gain = -1;\n        for (i32 c = 0; c < nc; ++c) {")],
    "gain_cap_off_by_one": [("if (gain > 0 && size[u] + size[r] <= cap &&", "if (gain > 0 && size[u] + size[r] < cap &&")],
    "gain_ties_to_largest_root": [("(gain == best_gain && r < best))) {", "(gain == best_gain && r > best))) {")],
    "gain_m_instead_of_2m": [("const i64 gain = conn[r] * M2 - deg[u] * deg[r];", "const i64 gain = conn[r] * (M2 / 2) - deg[u] * deg[r];")],
    "gain_visit_in_id_order": [("    if (x->deg != y->deg) return (x->deg > y->deg) - (x->deg < y->deg);\n", "")],
    "gain_visit_in_descending_degree": [("    if (x->deg != y->deg) return (x->deg > y->deg) - (x->deg < y->deg);", "    if (x->deg != y->deg) return (x->deg < y->deg) - (x->deg > y->deg);")],
    "gain_smallest_gain_wins": [("(gain > best_gain || (gain == best_gain && r < best))) {", "(best < 0 || gain < best_gain || (gain == best_gain && r < best))) {")],
}


def _build(tmp_path, name, patches):
    text = open(SRC).read()
    for old, new in patches:
        assert text.count(old) == 1, f"{name}: the oracle no longer contains exactly one {old!r}"
        text = text.replace(old, new)
    c = tmp_path / (name + ".c")
    so = tmp_path / (name + ".so")
    c.write_text(text)
    subprocess.check_call(["gcc", "-O1", "-fPIC", "-shared", "-std=c11", "-o", str(so), str(c), "-lm"])
    lib = ctypes.CDLL(str(so))
    lib.orc_reorder_method.restype = ctypes.c_int

    def reorder(rowptr, colidx, *, block_cap=128, min_block=16, sweeps=8, max_levels=12, order_levels=0, method=0):
        rowptr = np.ascontiguousarray(rowptr, np.int32)
        colidx = np.ascontiguousarray(colidx, np.int32)
        n = rowptr.size - 1
        perm, iperm, comm = (np.empty(n, np.int32) for _ in range(3))
        blk = np.empty(n + 1, np.int32)
        nb = ctypes.c_int32(0)
        ptr = lambda a: a.ctypes.data_as(ctypes.c_void_p)
        rc = lib.orc_reorder_method(ctypes.c_int64(n), ptr(rowptr), ptr(colidx), ctypes.c_int32(method), ctypes.c_int32(block_cap),
                             ctypes.c_int32(min_block), ctypes.c_int32(sweeps), ctypes.c_int32(max_levels),
                             ctypes.c_int32(order_levels), ptr(perm), ptr(iperm), ptr(blk), ctypes.byref(nb),
                             ptr(comm))
        assert rc == 0
        return SimpleNamespace(perm=perm, iperm=iperm, blk_ptr=blk[: nb.value + 1].copy(), comm=comm)

    return reorder


def test_unpatched_copy_passes_every_trace(tmp_path):
    assert failing_reorder_traces(_build(tmp_path, "unpatched", [])) == []


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_caught_by_a_hand_trace(tmp_path, name):
    failing = failing_reorder_traces(_build(tmp_path, name, MUTANTS[name]))
    assert failing, f"no hand-traced case notices the planted mistake '{name}'"
