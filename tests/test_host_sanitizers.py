"""The host plan code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

api.cpp, reorder.cpp and decompose.cpp are compiled as a plain host program with
-fsanitize=address,undefined (tests/sanitizer/host_stubs.cpp stands in for the kernel launchers
and the HIP runtime, which AG_FLAG_HOST_ONLY plans never reach) and driven through the C ABI on
six matrices, three block caps and both community-detection methods.  Any out-of-bounds access,
undefined behaviour or leak fails the test.
"""
import os
import subprocess

import numpy as np
import pytest

from ag_inputs import (config_graph, directed_random, from_edges, gcn_normalise, mixed_density,
                       planted_partition)

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2305_17408_amd", "csrc")
HERE = os.path.join(ROOT, "tests", "sanitizer")


def _compiler():
    for c in ("/opt/rocm/lib/llvm/bin/clang++", "/opt/rocm/llvm/bin/clang++", "g++"):
        if os.path.sep not in c or os.path.exists(c):
            return c
    return "g++"


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    d = tmp_path_factory.mktemp("san")
    exe = str(d / "driver")
    srcs = [os.path.join(CSRC, f) for f in ("api.cpp", "reorder.cpp", "decompose.cpp")]
    srcs += [os.path.join(HERE, "host_stubs.cpp"), os.path.join(HERE, "driver.cpp")]
    cmd = [_compiler(), "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-D__HIP_PLATFORM_AMD__", "-I", "/opt/rocm/include",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", exe, *srcs, "-lpthread"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
    return exe


def test_host_plan_code_is_clean_under_asan_and_ubsan(driver, tmp_path):
    graphs = {
        "sbm_weighted": config_graph(0),                                  # symmetric, GCN-normalised
        "directed": directed_random(1500, 3.0, 11),                       # non-symmetric pattern and values
        "powerlaw": config_graph(2, scale=1 / 64),                        # long rows, random block sizes
        "dense_blocks": mixed_density(12, 128, 0.3, 6, 0.02, 13),         # dense-class blocks, unit weights
        "small_caps": gcn_normalise(planted_partition(30, 16, 6, 0.8, 3)),
        "edgeless": from_edges(40, np.empty(0, int), np.empty(0, int), self_loops=False),
    }
    args = []
    for name, g in graphs.items():
        rp, ci, va = (str(tmp_path / f"{name}.{ext}") for ext in ("rowptr", "col", "val"))
        np.ascontiguousarray(g.rowptr, np.int32).tofile(rp)
        np.ascontiguousarray(g.colidx, np.int32).tofile(ci)
        if g.vals is not None:
            np.ascontiguousarray(g.vals, np.float32).tofile(va)
        args += [rp, ci, va]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([driver, *args], capture_output=True, text=True, env=env, timeout=600)
    out = r.stdout + r.stderr
    assert r.returncode == 0, out[-4000:]
    assert "AddressSanitizer" not in out and "runtime error" not in out and "LeakSanitizer" not in out, out[-4000:]
    assert out.count(" method ") == 6 * 2 * 3
