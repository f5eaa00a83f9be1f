"""The adaptive selector's state machine (paper Sec. 3.3) driven with made-up timings on the CPU.

csrc/selector.h is host-only logic; a few extern "C" shims around it are compiled with g++ into a
scratch library and called through ctypes.  No GPU, no HIP.
"""
import ctypes as C
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

SHIM = r"""
#include "selector.h"
using namespace ag;
extern "C" {
Selector *sel_new(const int *ncand, const int *forced) {
    Selector *s = new Selector();
    s->reset(false);
    for (int c = 0; c < AG_NUM_CLS; ++c) { s->ncand[c] = ncand[c]; s->forced[c] = forced[c]; }
    return s;
}
void sel_free(Selector *s) { delete s; }
int sel_next(Selector *s, int *k) { return selector_next(*s, k) ? 1 : 0; }
void sel_record(Selector *s, int trials, const int *k, const float *ms) { selector_record(*s, trials, k, ms); }
int sel_phase(const Selector *s) { return s->phase; }
float sel_median(const Selector *s, int c, int k) { return s->median_ms[c][k]; }
int sel_nsamples(const Selector *s, int c, int k) { return s->nsamples[c][k]; }
}
"""


@pytest.fixture(scope="module")
def shim(tmp_path_factory):
    d = tmp_path_factory.mktemp("selector")
    src, so = d / "shim.cpp", d / "libshim.so"
    src.write_text(SHIM)
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-fPIC", "-shared", "-I", os.path.join(ROOT, "include"),
                           "-I", os.path.join(ROOT, "paper_2305_17408_amd", "csrc"), "-o", str(so), str(src)])
    L = C.CDLL(str(so))
    L.sel_new.restype = C.c_void_p
    L.sel_new.argtypes = [C.POINTER(C.c_int), C.POINTER(C.c_int)]
    L.sel_free.argtypes = [C.c_void_p]
    L.sel_next.argtypes = [C.c_void_p, C.POINTER(C.c_int)]
    L.sel_record.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_float)]
    L.sel_phase.argtypes = [C.c_void_p]
    L.sel_median.argtypes = [C.c_void_p, C.c_int, C.c_int]
    L.sel_median.restype = C.c_float
    L.sel_nsamples.argtypes = [C.c_void_p, C.c_int, C.c_int]
    return L


def run(L, ncand, forced, timing, trials=3, limit=200):
    """Drive the selector to its frozen state.  timing(k, rep_index_of_this_candidate) -> the four
    intervals of a trial call with kernel ids k.  Returns (choice, trial log, handle-reading fn)."""
    s = L.sel_new((C.c_int * 4)(*ncand), (C.c_int * 4)(*forced))
    log, seen = [], {}
    k = (C.c_int * 4)()
    for _ in range(limit):
        if not L.sel_next(s, k):
            break
        key = (L.sel_phase(s), tuple(k))
        seen[key] = seen.get(key, 0) + 1
        ms = timing(tuple(k), seen[key] - 1, L.sel_phase(s))
        log.append((L.sel_phase(s), tuple(k), seen[key] - 1))
        L.sel_record(s, trials, k, (C.c_float * 4)(*ms))
    else:
        raise AssertionError("selector did not freeze")
    choice = tuple(k)
    med = {(c, i): L.sel_median(s, c, i) for c in range(4) for i in range(4)}
    ns = {(c, i): L.sel_nsamples(s, c, i) for c in range(4) for i in range(4)}
    assert L.sel_phase(s) == 2
    L.sel_free(s)
    return choice, log, med, ns


def test_cold_warm_up_does_not_discard_the_faster_candidate(shim):
    # remainder candidates: 0 takes 10 us; 1 takes 5 us but its first (cold) launch 500 us; 2 takes 8 us
    def timing(k, rep, phase):
        if phase == 0:
            r = {0: 0.010, 1: 0.500 if rep == 0 else 0.005, 2: 0.008}[k[2]]
            return (0.001, 0.001, r, r + 0.002)
        return (0, 0, 0, {0: 0.02, 1: 0.03, 2: 0.04, 3: 0.05}[k[3]])
    choice, log, med, ns = run(shim, (1, 1, 3, 4), (-1, -1, -1, -1), timing)
    assert choice[2] == 1                          # judged on warm repetitions only
    assert ns[(2, 1)] == 3 and abs(med[(2, 1)] - 0.005) < 1e-9
    assert choice[3] == 0


def test_hopeless_candidate_is_abandoned_after_its_first_timed_repetition(shim):
    def timing(k, rep, phase):
        if phase == 0:
            r = {0: 0.010, 1: 0.011, 2: 0.300}[k[2]]          # candidate 2 is 30x slower
            return (0.001, 0.001, r, r + 0.002)
        return (0, 0, 0, 0.02 + 0.01 * k[3])
    choice, log, med, ns = run(shim, (1, 1, 3, 4), (-1, -1, -1, -1), timing)
    calls_c2 = [x for x in log if x[0] == 0 and x[1][2] == 2]
    assert len(calls_c2) == 2                      # warm-up + one timed repetition, then dropped
    assert ns[(2, 2)] == 1 and abs(med[(2, 2)] - 0.300) < 1e-6   # a warm sample, not the cold one
    assert choice[2] == 0
    assert len([x for x in log if x[0] == 0 and x[1][2] == 0]) == 4


def test_ties_go_to_the_lowest_id_and_unmeasured_candidates_never_win(shim):
    def timing(k, rep, phase):
        return (0.01, 0.01, 0.01, 0.03)
    choice, log, med, ns = run(shim, (3, 1, 3, 4), (-1, -1, -1, -1), timing)
    assert choice == (0, 0, 0, 0)
    # phase 0 runs max(ncand) = 3 candidates x (1 + 3) calls, phase 1 four compositions x 4 calls
    assert len(log) == 3 * 4 + 4 * 4
    assert med[(1, 1)] < 0                         # the sparse class has one candidate: nothing else measured


def test_forced_classes_are_not_tried(shim):
    def timing(k, rep, phase):
        return (0.01, 0.01, 0.01, 0.03)
    choice, log, _, _ = run(shim, (3, 1, 3, 4), (2, 0, 1, 1), timing)
    assert log == [] and choice == (2, 0, 1, 1)
    choice, log, _, _ = run(shim, (3, 1, 3, 4), (2, 0, 1, -1), timing)
    assert all(ph == 1 and k[:3] == (2, 0, 1) for ph, k, _ in log) and len(log) == 16


def test_the_dense_class_and_the_remainder_are_judged_independently(shim):
    # dense candidate 2 is fastest for its class, remainder candidate 0 for its own
    def timing(k, rep, phase):
        if phase == 0:
            d = {0: 0.09, 1: 0.06, 2: 0.03}[k[0]]
            r = {0: 0.10, 1: 0.12, 2: 0.35}[k[2]]
            return (d, 0.01, r, d + r + 0.01)
        return (0, 0, 0, {0: 0.20, 1: 0.15, 2: 0.30, 3: 0.31}[k[3]])
    choice, log, med, ns = run(shim, (3, 1, 3, 4), (-1, -1, -1, -1), timing)
    assert choice == (2, 0, 0, 1)
    # candidate index 2 pairs dense 2 with remainder 2; the remainder is slow there but the dense
    # class is not, so the pair is measured in full
    assert ns[(0, 2)] == 3 and ns[(2, 2)] == 3
    # the composition trials ran with the winners of the class trials
    assert all(k[:3] == (2, 0, 0) for ph, k, _ in log if ph == 1)
