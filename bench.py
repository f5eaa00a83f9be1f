#!/usr/bin/env python3
"""Benchmark of the aggregation hot path on one MI355X.

A step = one forward aggregation Y = A.H plus one backward aggregation dH = A^T.G on the
workload's graph and feature width, through the C ABI (ag_aggregate / ag_aggregate_t) on
plan-ordered features resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config IDX] [--no-cpu] [--no-gcn]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
AG_MIN_OWN = 256          # AG_MIN_BLOCKS_OWN_LAUNCH of the C header


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes(st, F, compose, cls, dense_kernel=0):
    """Algorithmic HBM bytes of one launch of the kernel(s) of class `cls` (0 dense-class blocks,
    1 sparse-class blocks, 2 remainder / one CSR).

    Block kernels: the class's topology once (block CSR with one-byte columns, or for the dense
    kernels a 2 KB bit map per block plus a 64 KB value tile if weighted), every feature row of
    the class once, every output row once; fused, also the remainder CSR of those rows and one
    feature-row fetch per remainder entry (the sources of the inter-community subgraph have no
    locality by construction).  Remainder kernel (SPLIT): its CSR once, one fetch per entry, one
    write of every output row plus the read of the block rows it accumulates onto.
    """
    n, nbr = st["n"], st["n_block_rows"]
    wbytes = 0 if st["unit_weights"] else 4
    row = 4 * F
    if cls == 2:
        if compose >= 2:                       # one CSR over everything
            return 4 * (n + 1) + (4 + wbytes) * st["nnz"] + row * (n + st["nnz_inter"]) + row * n
        if compose == 1:                       # tail rows only; block rows were fused
            tail = st["nnz_inter"] - st["nnz_inter_block_rows"]
            return 4 * (n - nbr + 1) + (4 + wbytes) * tail + row * tail + row * (n - nbr)
        return 4 * (n + 1) + (4 + wbytes) * st["nnz_inter"] + row * st["nnz_inter"] + row * n + row * nbr
    # does the dense class run its own (dense) kernel?  In the fused composition only from a minimum size on.
    dense_own = dense_kernel != 0 and st["n_dense_blocks"] >= (AG_MIN_OWN if compose == 1 else 1)
    d_rows, d_intra, d_inter = st["dense_rows"], st["nnz_intra_dense"], st["nnz_inter_dense_rows"]
    if cls == 0 and dense_own:
        rows, inter = d_rows, d_inter
        topo = st["n_dense_blocks"] * (2048 + (0 if st["unit_weights"] else 65536))
    else:
        if compose == 1 and not dense_own:     # one fused kernel over all blocks
            rows, intra, inter = nbr, st["nnz_intra"], st["nnz_inter_block_rows"]
        elif cls == 0:
            rows, intra, inter = d_rows, d_intra, d_inter
        else:
            rows, intra, inter = nbr - d_rows, st["nnz_intra"] - d_intra, st["nnz_inter_block_rows"] - d_inter
        topo = 4 * (rows + 1) + (1 + wbytes) * intra
    total = topo + 2 * row * rows
    if compose == 1:
        total += 4 * (rows + 1) + (4 + wbytes) * inter + row * inter
    return total


def measured_traffic(config, F, choice):
    """(HBM bytes per launch of the dominant kernel, where the figure comes from) from the committed
    rocprofv3 --pmc summaries, for exactly this workload, width and kernel choice [dense-class kernel,
    sparse-class kernel, remainder kernel, composition]; (None, reason) when no committed counter run
    covers that choice: the figure is measured in separate profiler runs, not in this run."""
    try:
        for line in open(os.path.join(ROOT, "profiles", "hbm_traffic_bytes.txt")):
            t = line.split()
            if len(t) >= 8 and not line.startswith("#") and [int(x) for x in t[:6]] == [config, F] + list(choice):
                return int(t[6]), f"profiles/{t[8] if len(t) > 8 else 'hbm_traffic_bytes.txt'}, rocprofv3 --pmc runs of {t[7]}"
    except (OSError, ValueError):
        pass
    return None, "no committed counter run for this workload, width and kernel choice"


def brief(index, steps):
    """Short measurement of another workload: ms per aggregation, selector timings, plan cost."""
    import torch
    import paper_2305_17408_amd as ag
    from ag_inputs import config_graph, CONFIGS, features
    cfg = CONFIGS[index]
    F = cfg["F"]
    g = config_graph(index)
    t0 = time.time()
    plan = ag.ag_plan_create(g.rowptr, g.colidx, g.vals, g.n, F, layout=ag.AG_LAYOUT_REORDERED)
    t_plan = time.time() - t0
    st = ag.ag_plan_stats(plan)
    H = torch.from_numpy(features(g.n, F, 7)).cuda()
    G = torch.from_numpy(features(g.n, F, 8)).cuda()
    Y, dH = torch.empty_like(H), torch.empty_like(H)
    n = 0
    while n < 200 and not (ag.ag_plan_selector_info(plan, 0)["frozen"] and ag.ag_plan_selector_info(plan, 1)["frozen"]):
        ag.ag_aggregate(plan, H, Y)
        ag.ag_aggregate_t(plan, G, dH)
        n += 1
    for _ in range(5):
        ag.ag_aggregate(plan, H, Y)
        ag.ag_aggregate_t(plan, G, dH)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        ag.ag_aggregate(plan, H, Y)
        ag.ag_aggregate_t(plan, G, dH)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    sel = ag.ag_plan_selector_info(plan, 0)
    ag.ag_plan_destroy(plan)
    compulsory = 2 * (4 * (g.n + 1) + (4 + (0 if g.vals is None else 4)) * g.nnz + 8 * g.n * F)
    t = sel["trial_ms"]
    log(f"[bench] configs[{index}] {cfg['name']}: {ms:.4f} ms/step, choice {sel['choice']}")
    return {"workload": f"configs[{index}] {cfg['name']}", "n": g.n, "nnz": g.nnz, "F": F,
            "ms_per_step": round(ms, 5), "gflops": round(4.0 * g.nnz * F / ms / 1e6, 1),
            "effective_hbm_gbs": round(compulsory / ms / 1e6, 1), "selector_choice_fwd": sel["choice"],
            "trial_ms_fwd": {"dense_class_bsp_f32_bf16x3": [round(x, 5) for x in t[0][:3]], "sparse_class": round(t[1][0], 5),
                             "remainder": [round(x, 5) for x in t[2][:3]],
                             "compose_split_fused_full_fullwide": [round(x, 5) for x in t[3][:4]]},
            "plan_create_s": round(t_plan, 2), "nnz_intra": st["nnz_intra"], "nnz_inter": st["nnz_inter"],
            "n_blocks": st["n_blocks"], "n_dense_blocks": st["n_dense_blocks"], "n_long_rows": st["n_long_rows"],
            "density_full": st["density_full"], "density_intra": st["density_intra"],
            "density_inter": st["density_inter"], "plan_device_bytes": st["device_bytes"]}


def captured_intra(g, st):
    """Share of the graph's edges that the reordering keeps inside diagonal blocks, next to the share
    the generator planted inside its communities (self-loops left out on both sides)."""
    edges = g.meta.get("edges")
    if not edges:
        return {}
    got = (st["nnz_intra"] - st["n_block_rows"]) / 2.0 / edges
    planted = g.meta.get("planted_intra_frac", 0.0)
    return {"intra_edge_frac_captured": round(got, 4), "intra_edge_frac_planted": round(planted, 4),
            "captured_over_planted": round(got / planted, 4) if planted > 0 else None}


def event_medians(fn, calls):
    """Median and spread (ms) of `calls` individually timed launches of fn() with events on the
    current stream (the stream the binding launches on)."""
    import torch
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(calls)]
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    t = sorted(a.elapsed_time(b) for a, b in ev)
    return t[len(t) // 2], t[0], t[-1]


def pin(ag, plan, compose, dense, rem):
    for d in (0, 1):
        ag.ag_plan_force_kernels(plan, ag.AG_CLS_COMPOSE, d, compose)
        ag.ag_plan_force_kernels(plan, ag.AG_CLS_BLOCKS_DENSE, d, dense)
        ag.ag_plan_force_kernels(plan, ag.AG_CLS_BLOCKS_SPARSE, d, 0)
        ag.ag_plan_force_kernels(plan, ag.AG_CLS_REMAINDER, d, rem)


def unpin(ag, plan):
    for d in (0, 1):
        for c in range(4):
            ag.ag_plan_force_kernels(plan, c, d, -1)


def adaptive_vs_single_format(index, calls):
    """The breakdown of the paper's Sec. 6.2 on the mixed-density workload, ms per step (forward +
    backward, median of `calls` steps timed with events):
      single format (one kernel over the whole reordered matrix, O1 of the paper):
        one_csr_narrow / one_csr_wide   the CSR kernel with one / several lane groups per row
      static subgraph-level kernel sets (no selector; O2 of the paper is the first one):
        csr_intra+coo_inter             block-sparse kernel for every block, COO kernel for the remainder
        csr_intra+csr_inter             block-sparse kernel for every block, CSR remainder, best composition
        dense_f32+csr_inter             fp32 MFMA kernel for every block of >= 32 rows (plan with
                                        dense_density ~ 0), CSR remainder, best composition
        dense_bf16x3+csr_inter          the same on the bf16 MFMA form (unit-weight matrices)
      adaptive (O3)                     what the selector froze on
    The adaptive set can at best equal the fastest static set (it is one of them, found by timing);
    the target is its ratio to the best single-format kernel."""
    import torch
    import paper_2305_17408_amd as ag
    from ag_inputs import config_graph, CONFIGS, features
    cfg = CONFIGS[index]
    F = cfg["F"]
    g = config_graph(index)
    H = torch.from_numpy(features(g.n, F, 7)).cuda()
    G = torch.from_numpy(features(g.n, F, 8)).cuda()
    Y, dH = torch.empty_like(H), torch.empty_like(H)
    plan = ag.ag_plan_create(g.rowptr, g.colidx, g.vals, g.n, F, layout=ag.AG_LAYOUT_REORDERED)
    st = ag.ag_plan_stats(plan)

    def step(p):
        ag.ag_aggregate(p, H, Y)
        ag.ag_aggregate_t(p, G, dH)

    def timed(p, k=calls):
        for _ in range(3):
            step(p)
        return event_medians(lambda: step(p), k)[0]

    n = 0
    while n < 200 and not (ag.ag_plan_selector_info(plan, 0)["frozen"] and ag.ag_plan_selector_info(plan, 1)["frozen"]):
        step(plan)
        n += 1
    choice = ag.ag_plan_selector_info(plan, 0)["choice"]
    adaptive = timed(plan)
    single, static = {}, {}
    for name, (c, r) in {"one_csr_narrow": (2, 0), "one_csr_wide": (3, 1)}.items():
        pin(ag, plan, c, 0, r)
        single[name] = timed(plan)
    pin(ag, plan, 0, 0, 2)
    static["csr_intra+coo_inter"] = timed(plan, 10)
    best = None
    for c in (0, 1):
        pin(ag, plan, c, 0, 0)
        t = timed(plan)
        best = t if best is None else min(best, t)
    static["csr_intra+csr_inter"] = best
    ag.ag_plan_destroy(plan)
    plan = ag.ag_plan_create(g.rowptr, g.colidx, g.vals, g.n, F, layout=ag.AG_LAYOUT_REORDERED, dense_density=1e-9)
    st2 = ag.ag_plan_stats(plan)
    kinds = {"dense_f32+csr_inter": 1}
    if g.vals is None:
        kinds["dense_bf16x3+csr_inter"] = 2
    for name, k in kinds.items():
        best = None
        for c in (0, 1):
            pin(ag, plan, c, k, 0)
            t = timed(plan)
            best = t if best is None else min(best, t)
        static[name] = best
    ag.ag_plan_destroy(plan)
    best_single = min(single, key=single.get)
    best_static = min(static, key=static.get)
    out = {"workload": f"configs[{index}] {cfg['name']}: N={g.n}, nnz={g.nnz}, F={F}, forward + backward",
           "calls": calls, "unit": "ms per step (median)",
           "adaptive_ms": round(adaptive, 5), "adaptive_choice_fwd": choice,
           "single_format_ms": {k: round(v, 5) for k, v in single.items()},
           "static_sets_ms": {k: round(v, 5) for k, v in static.items()},
           "best_single_format": best_single,
           "speedup_over_best_single_format": round(single[best_single] / adaptive, 3),
           "best_static_set": best_static,
           "adaptive_over_best_static_set": round(adaptive / static[best_static], 3),
           "blocks": st["n_blocks"], "dense_class_blocks": st["n_dense_blocks"],
           "dense_class_blocks_in_all_dense_plan": st2["n_dense_blocks"]}
    log(f"[bench] adaptive vs single format: {out}")
    return out


def density_sweep():
    """Kernel timings over a sweep of subgraph densities (the shape of the paper's format-versus-
    density figure in Sec. 2.1, on synthetic graphs): (a) diagonal blocks of 128 vertices whose
    density is swept, every block put in the dense class so that all three block kernels are timed;
    (b) a block-less graph whose average degree is swept, timing the CSR and COO remainder kernels.
    Times are the selector's median trial times (HIP events) of the forward direction, in ms."""
    import torch
    import paper_2305_17408_amd as ag
    from ag_inputs import mixed_density, planted_partition, features
    F = 32

    def trials(g, **opts):
        plan = ag.ag_plan_create(g.rowptr, g.colidx, g.vals, g.n, F, layout=ag.AG_LAYOUT_REORDERED, trials=5, **opts)
        H = torch.from_numpy(features(g.n, F, 7)).cuda()
        Y = torch.empty_like(H)
        n = 0
        while n < 200 and not ag.ag_plan_selector_info(plan, 0)["frozen"]:
            ag.ag_aggregate(plan, H, Y)
            n += 1
        torch.cuda.synchronize()
        info, st = ag.ag_plan_selector_info(plan, 0), ag.ag_plan_stats(plan)
        ag.ag_plan_destroy(plan)
        return info, st

    blocks = []
    for p in (0.005, 0.01, 0.02, 0.05, 0.1, 0.2, 0.3, 0.5, 0.8):
        g = mixed_density(1024, 128, p, 6, 0.02, 4000 + int(p * 1000))
        info, st = trials(g, dense_density=1e-9)
        t = info["trial_ms"]
        row = {"block_density": p, "n": g.n, "nnz": g.nnz, "n_dense_class_blocks": st["n_dense_blocks"],
               "density_intra": round(st["density_intra"], 4),
               "block_sparse_ms": round(t[0][0], 5), "dense_f32_ms": round(t[0][1], 5),
               "dense_bf16x3_ms": round(t[0][2], 5), "choice": info["choice"]}
        log(f"[sweep] {row}")
        blocks.append(row)
    rem = []
    for deg in (0.125, 0.25, 0.5, 1, 2, 4, 8, 16):
        g = planted_partition(2048, 128, deg, 0.0, 5000 + int(deg * 8))
        info, st = trials(g, min_block=129)
        t = info["trial_ms"]
        row = {"avg_degree": deg, "n": g.n, "nnz": g.nnz, "density": st["density_full"],
               "csr_narrow_ms": round(t[2][0], 5), "csr_wide_ms": round(t[2][1], 5), "coo_ms": round(t[2][2], 5),
               "choice": info["choice"]}
        log(f"[sweep] {row}")
        rem.append(row)
    # (c) R-MAT graphs of 19 717 vertices over a density sweep (the graphs of the paper's format-versus-
    # density figure, Sec. 2.1): whole-graph kernels (no blocks: min_block above the cap) and the
    # adaptive decomposition on the same graph
    from ag_inputs import rmat
    n = 19717
    rm = []
    for dens in (1e-5, 3e-5, 1e-4, 3e-4, 1e-3, 3e-3, 1e-2, 3e-2):
        g = rmat(n, int(dens * n * n / 2), 6000 + int(dens * 1e6))
        info, st = trials(g, min_block=129)
        t = info["trial_ms"]
        info2, st2 = trials(g)
        t2 = info2["trial_ms"][3]
        row = {"density": dens, "n": g.n, "nnz": g.nnz, "max_degree": int(np.diff(g.rowptr).max()),
               "csr_narrow_ms": round(t[2][0], 5), "csr_wide_ms": round(t[2][1], 5), "coo_ms": round(t[2][2], 5),
               "decomposed_split_ms": round(t2[0], 5), "decomposed_fused_ms": round(t2[1], 5),
               "blocks": st2["n_blocks"], "dense_class_blocks": st2["n_dense_blocks"],
               "intra_share": round(st2["nnz_intra"] / max(1, st2["nnz"]), 4), "adaptive_choice": info2["choice"]}
        log(f"[sweep] {row}")
        rm.append(row)
    return {"F": F, "block_kernels_vs_block_density": blocks, "remainder_kernels_vs_degree": rem,
            "rmat_19717_vs_density": rm}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--config", type=int, default=3, help="index of the benchmark workload (0-based, see ag_inputs.CONFIGS)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-gcn", action="store_true", help="skip the GCN training-step timing")
    ap.add_argument("--no-mixed", action="store_true",
                    help="skip the adaptive-versus-single-format comparison on the mixed-density workload (configs[4])")
    ap.add_argument("--all-configs", action="store_true",
                    help="also time the other four workloads (short runs) and add them under 'other_workloads'")
    ap.add_argument("--width", type=int, default=0,
                    help="feature width F to run the workload's graph with instead of its own (0 = the workload's width)")
    ap.add_argument("--pin", default="",
                    help="pin the kernels instead of letting the selector choose: COMPOSE[,DENSE[,REMAINDER]] with "
                         "COMPOSE in split|fused|full|full_wide, DENSE in 0|1|2 (block-sparse, fp32 MFMA, bf16x3 MFMA), "
                         "REMAINDER in 0|1|2 (CSR narrow, CSR wide, COO); for profiling one kernel set in isolation")
    ap.add_argument("--density-sweep", action="store_true",
                    help="instead of the benchmark, time every kernel candidate over a sweep of subgraph densities")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (the path is single-GPU by design); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    if args.density_sweep:
        print(json.dumps({"density_sweep": density_sweep()}), flush=True)
        return

    import torch
    import paper_2305_17408_amd as ag
    from ag_inputs import config_graph, CONFIGS, features, glorot_uniform, labels

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    cfg = CONFIGS[args.config]
    F = args.width if args.width > 0 else cfg["F"]
    t0 = time.time()
    g = config_graph(args.config)
    log(f"[bench] graph {cfg['name']}: n={g.n} nnz={g.nnz} F={F} ({time.time() - t0:.1f}s)")
    t0 = time.time()
    plan = ag.ag_plan_create(g.rowptr, g.colidx, g.vals, g.n, F, layout=ag.AG_LAYOUT_REORDERED)
    t_plan = time.time() - t0
    st = ag.ag_plan_stats(plan)
    log(f"[bench] plan: {t_plan:.1f}s blocks={st['n_blocks']} dense={st['n_dense_blocks']} "
        f"intra={st['nnz_intra']} inter={st['nnz_inter']} long_rows={st['n_long_rows']}")
    # the same plan from its saved reordering (what a second training on the graph pays)
    ex = ag.ag_plan_export(plan)
    saved = (ex["perm"].copy(), ex["blk_ptr"].copy())
    t0 = time.time()
    plan2 = ag.ag_plan_create(g.rowptr, g.colidx, g.vals, g.n, F, layout=ag.AG_LAYOUT_REORDERED, reuse=saved)
    t_plan_reuse = time.time() - t0
    ag.ag_plan_destroy(plan2)
    log(f"[bench] plan from a saved reordering: {t_plan_reuse:.2f}s")

    H = torch.from_numpy(features(g.n, F, 7)).to(dev)
    G = torch.from_numpy(features(g.n, F, 8)).to(dev)
    Hp, Gp = torch.empty_like(H), torch.empty_like(G)
    ag.ag_permute_rows(plan, H, Hp, F, False)
    ag.ag_permute_rows(plan, G, Gp, F, False)
    Y, dH = torch.empty_like(H), torch.empty_like(H)
    torch.cuda.synchronize()
    if args.pin:
        t = args.pin.split(",")
        pin(ag, plan, {"split": 0, "fused": 1, "full": 2, "full_wide": 3}[t[0]], int(t[1]) if len(t) > 1 else 0,
            int(t[2]) if len(t) > 2 else 0)

    def step():
        ag.ag_aggregate(plan, Hp, Y)
        ag.ag_aggregate_t(plan, Gp, dH)

    # selector trials belong to plan set-up ("first iterations"): run until both directions froze
    sel_calls = 0
    t0 = time.time()
    while not (ag.ag_plan_selector_info(plan, 0)["frozen"] and ag.ag_plan_selector_info(plan, 1)["frozen"]):
        step()
        sel_calls += 1
        if sel_calls > 200:
            break
    torch.cuda.synchronize()
    t_sel = time.time() - t0
    sel = [ag.ag_plan_selector_info(plan, d) for d in (0, 1)]
    log(f"[bench] selector froze after {sel_calls} steps ({t_sel:.2f}s): fwd {sel[0]['choice']} bwd {sel[1]['choice']}")

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_step = dt * 1e3 / args.steps
    flop = 4.0 * g.nnz * F
    gflops = flop / (ms_step * 1e-3) / 1e9
    compulsory = 2 * (4 * (g.n + 1) + (4 + (0 if g.vals is None else 4)) * g.nnz + 8 * g.n * F)
    log(f"[bench] {ms_step:.4f} ms/step  {gflops:.1f} GFLOP/s  effective {compulsory / ms_step / 1e6:.1f} GB/s")
    # forward, backward and whole steps timed one by one with events: medians of >= 50 calls
    ncall = max(50, args.steps)
    med = {"calls": ncall}
    for name, fn in (("forward", lambda: ag.ag_aggregate(plan, Hp, Y)),
                     ("backward", lambda: ag.ag_aggregate_t(plan, Gp, dH)), ("step", step)):
        m, lo, hi = event_medians(fn, ncall)
        med[name] = {"median_ms": round(m, 5), "min_ms": round(lo, 5), "max_ms": round(hi, 5)}
    log(f"[bench] medians over {ncall} calls: {med}")

    # the same steps again with HIP events around every subgraph kernel (roofline figures)
    ag.ag_plan_set_profiling(plan, True)
    for _ in range(args.steps):
        step()
    prof = [ag.ag_plan_profile(plan, d) for d in (0, 1)]
    ag.ag_plan_set_profiling(plan, False)
    compose = prof[0]["compose"]
    dense_own = sel[0]["choice"][0] != 0 and st["n_dense_blocks"] >= (AG_MIN_OWN if compose == 1 else 1)
    if compose == 1 and dense_own:
        cls_names = {0: "fused dense-class kernel (MFMA + the rows' remainder)",
                     1: "fused sparse-class kernel (intra from LDS + the rows' remainder)",
                     2: "tail rows + long-row segments"}
    elif compose == 1:
        cls_names = {0: "fused block kernel (all blocks: intra from LDS + their remainder rows)",
                     1: "(unused)", 2: "tail rows + long-row segments"}
    elif compose >= 2:
        cls_names = {0: "(unused)", 1: "(unused)", 2: "one CSR over the whole reordered matrix"}
    else:
        cls_names = {0: "dense-class blocks", 1: "sparse-class blocks", 2: "remainder CSR"}
    per_class = {}
    for c in range(3):
        ms = sum(p["class_ms"][c] for p in prof)
        calls = sum(p["calls"] for p in prof)
        per_class[c] = ms / max(1, calls)
    dom = max(per_class, key=per_class.get)
    dense_names = {1: "k_block_dense", 2: "k_block_dense_bf16x3"}
    if dom == 2:
        dom_name = "k_csr_rows (+ long-row segments)"
    elif dom == 0 and dense_own:
        dom_name = dense_names[sel[0]["choice"][0]] + ("<..., FUSED=true>" if compose == 1 else "")
    else:
        dom_name = "k_block_sparse" + ("<..., FUSED=true>" if compose == 1 else "")
    abytes = algorithmic_bytes(st, F, compose, dom, sel[0]["choice"][0])
    achieved = abytes / (per_class[dom] * 1e-3) / 1e9 if per_class[dom] > 0 else 0.0
    traffic, traffic_source = measured_traffic(args.config, F, sel[0]["choice"])
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": traffic, "traffic_source": traffic_source,
                # the whole forward aggregation against the bytes no algorithm can avoid (every array once)
                "frac_compulsory": round(compulsory / 2 / (med["forward"]["median_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                "kernel": dom_name, "class": cls_names[dom], "avg_launch_ms": round(per_class[dom], 5),
                "algorithmic_bytes_per_launch": int(abytes),
                "per_class_ms": {cls_names[c]: round(per_class[c], 5) for c in per_class}}
    log(f"[bench] roofline: {roofline}")
    # the sparse-remainder kernel on its own: SPLIT composition pinned, HIP events around the remainder
    # kernel (class 2) over >= 20 aggregations per direction; afterwards the frozen choice is pinned back
    rem = {}
    if st["nnz_inter"] > 0 and not args.pin:
        pin(ag, plan, 0, 0, 0)
        for _ in range(3):
            step()
        ag.ag_plan_set_profiling(plan, True)
        for _ in range(max(20, args.steps // 2)):
            step()
        pr = [ag.ag_plan_profile(plan, d) for d in (0, 1)]
        ag.ag_plan_set_profiling(plan, False)
        for d in (0, 1):
            for c in range(4):
                ag.ag_plan_force_kernels(plan, c, d, sel[d]["choice"][c])
        rem_ms = sum(p["class_ms"][2] for p in pr) / max(1, sum(p["calls"] for p in pr))
        rem_bytes = algorithmic_bytes(st, F, 0, 2)
        rem_traffic, rem_src = measured_traffic(args.config, F, [0, 0, 0, 0])
        rem = {"kernel": "k_csr_rows (+ long-row segments) on the inter-community CSR, accumulating onto the block rows",
               "launches_timed": sum(p["calls"] for p in pr), "avg_launch_ms": round(rem_ms, 5),
               "traffic": rem_traffic, "traffic_source": rem_src,
               "frac": round(rem_traffic / (rem_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4) if (rem_traffic and rem_ms > 0) else None,
               "algorithmic_bytes_per_launch": int(rem_bytes),
               "algorithmic_frac": round(rem_bytes / (rem_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4) if rem_ms > 0 else None,
               "unit": "GB/s", "peak": HBM_PEAK_GBS,
               "note": "frac = committed counter traffic of this kernel / its launch time measured in this run / peak; "
                       "algorithmic_frac uses the no-reuse byte count instead"}
        log(f"[bench] remainder kernel alone: {rem}")
    remainder = rem
    compose_ms = dict(zip(("split", "fused", "full_csr", "full_csr_wide"), [round(t, 5) for t in sel[0]["trial_ms"][3][:4]]))

    out = {
        "metric": "aggregation GFLOP/s (fwd+bwd SpMM, fp32)", "value": round(gflops, 2), "unit": "GFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"configs[{args.config}] {cfg['name']}: N={g.n}, nnz={g.nnz}, F={F}, "
                               "one forward + one backward aggregation, plan-ordered features",
                   "n": g.n, "nnz": g.nnz, "F": F, "layout": "reordered"},
        "medians": med,
        "effective_hbm_gbs": round(compulsory / ms_step / 1e6, 1),
        "compulsory_bytes_per_step": int(compulsory),
        "plan_create_s": round(t_plan, 2), "plan_create_from_saved_reordering_s": round(t_plan_reuse, 2),
        "selector_steps": sel_calls, "selector_s": round(t_sel, 3),
        "selector_choice": {"fwd": sel[0]["choice"], "bwd": sel[1]["choice"]},
        "plan": {**{k: st[k] for k in ("n_blocks", "n_block_rows", "n_dense_blocks", "nnz_intra", "nnz_inter",
                                       "n_long_rows", "n_long_segments", "sec_reorder", "sec_split", "sec_build",
                                       "sec_upload", "device_bytes")},
                 **captured_intra(g, st)},
        "roofline": roofline,
        "remainder_path": remainder,
        "selector_trial_ms": {"compositions_fwd": compose_ms,
                              "dense_class_fwd": {"block_sparse": round(sel[0]["trial_ms"][0][0], 5),
                                                  "dense_mfma_f32": round(sel[0]["trial_ms"][0][1], 5),
                                                  "dense_mfma_bf16x3": round(sel[0]["trial_ms"][0][2], 5)}},
    }

    # the max aggregator (forward with argmax + adjoint) on the same graph and features
    if not args.no_gcn:
        arg = torch.empty(g.n, F, dtype=torch.int32, device=dev)
        for _ in range(3):
            ag.ag_aggregate_max(plan, Hp, Y, arg)
            ag.ag_aggregate_max_t(plan, Gp, arg, dH)
        torch.cuda.synchronize()
        k = max(5, args.steps // 5)
        t0 = time.perf_counter()
        for _ in range(k):
            ag.ag_aggregate_max(plan, Hp, Y, arg)
            ag.ag_aggregate_max_t(plan, Gp, arg, dH)
        torch.cuda.synchronize()
        out["max_aggregator_ms_per_step"] = round((time.perf_counter() - t0) * 1e3 / k, 4)
        log(f"[bench] max aggregator fwd+adjoint {out['max_aggregator_ms_per_step']} ms/step")
        del arg

    # ms per 2-layer GCN training step (only defined for the GCN workload)
    if not args.no_gcn and "hidden" in cfg and F == cfg["F"]:
        hid, ncls = cfg["hidden"], cfg["classes"]
        p_out = ag.ag_plan_clone_for_width(plan, ncls)
        t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        W1, W2 = t(glorot_uniform(F, hid, 21)), t(glorot_uniform(hid, ncls, 22))
        b1, b2 = torch.zeros(hid, device=dev), torch.zeros(ncls, device=dev)
        perm = ag.ag_plan_export(plan)["perm"]
        yl = t(labels(g.n, ncls, 23)[perm])
        dW1, db1 = torch.empty_like(W1), torch.empty_like(b1)
        dW2, db2 = torch.empty_like(W2), torch.empty_like(b2)
        loss = torch.empty(1, device=dev)
        ws = torch.empty(ag.ag_gcn_workspace_bytes(g.n, F, hid, ncls) // 4, device=dev)

        def gcn(stream=None):
            ag.ag_gcn_step(plan, p_out, f_in=F, hidden=hid, n_class=ncls, W1=W1, b1=b1, W2=W2, b2=b2,
                           dW1=dW1, db1=db1, dW2=dW2, db2=db2, loss=loss, logits=None, X=Hp, labels=yl,
                           workspace=ws, stream=stream)
        n_sel = 0
        while n_sel < 60 and not (ag.ag_plan_selector_info(p_out, 0)["frozen"]
                                  and ag.ag_plan_selector_info(p_out, 1)["frozen"]):
            gcn()
            n_sel += 1
        for _ in range(3):
            gcn()
        torch.cuda.synchronize()
        k = max(5, args.steps // 5)
        t0 = time.perf_counter()
        for _ in range(k):
            gcn()
        torch.cuda.synchronize()
        out["gcn_step_ms"] = round((time.perf_counter() - t0) * 1e3 / k, 4)
        out["gcn_loss"] = round(float(loss.item()), 6)
        log(f"[bench] GCN step {out['gcn_step_ms']} ms, loss {out['gcn_loss']}")
        # the same step recorded once into a HIP graph (both plans are frozen: a step only enqueues kernels)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                gcn(side)
        torch.cuda.current_stream().wait_stream(side)
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(k):
            graph.replay()
        torch.cuda.synchronize()
        out["gcn_step_hip_graph_ms"] = round((time.perf_counter() - t0) * 1e3 / k, 4)
        out["gcn_loss_hip_graph"] = round(float(loss.item()), 6)
        log(f"[bench] GCN step as a HIP graph {out['gcn_step_hip_graph_ms']} ms, loss {out['gcn_loss_hip_graph']}")
        del graph
        ag.ag_plan_destroy(p_out)

    # ms per 5-layer GIN training step (hidden 64, 16 classes) on the unit-weight GIN workload
    if not args.no_gcn and cfg.get("norm") == "unit" and F == cfg["F"]:
        widths = [F, 64, 64, 64, 64, 16]
        L = len(widths) - 1
        by_w = {F: plan}
        for w in widths:
            if w not in by_w:
                by_w[w] = ag.ag_plan_clone_for_width(plan, w)
        plans = [by_w[w] for w in widths]
        t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        Wd = [t(0.05 * glorot_uniform(widths[l], widths[l + 1], 31 + l)) for l in range(L)]   # keeps activations O(1)
        bd = [torch.zeros(widths[l + 1], device=dev) for l in range(L)]
        dWd, dbd = [torch.empty_like(w) for w in Wd], [torch.empty_like(b) for b in bd]
        perm = ag.ag_plan_export(plan)["perm"]
        yl = t(labels(g.n, widths[-1], 23)[perm])
        loss = torch.empty(1, device=dev)
        ws = torch.empty(ag.ag_gin_workspace_bytes(g.n, widths) // 4, device=dev)

        def gin():
            ag.ag_gin_step(plans, widths=widths, eps=0.0, W=Wd, b=bd, dW=dWd, db=dbd, loss=loss, logits=None,
                           X=Hp, labels=yl, workspace=ws)
        n_sel = 0
        while n_sel < 80 and not all(ag.ag_plan_selector_info(p, d)["frozen"] for p in by_w.values() for d in (0, 1)):
            gin()
            n_sel += 1
        for _ in range(3):
            gin()
        torch.cuda.synchronize()
        k = max(5, args.steps // 5)
        t0 = time.perf_counter()
        for _ in range(k):
            gin()
        torch.cuda.synchronize()
        out["gin_step_ms"] = round((time.perf_counter() - t0) * 1e3 / k, 4)
        out["gin_step_widths"] = widths
        out["gin_loss"] = round(float(loss.item()), 6)
        log(f"[bench] GIN step ({widths}) {out['gin_step_ms']} ms, loss {out['gin_loss']}")
        for w, p in by_w.items():
            if p is not plan:
                ag.ag_plan_destroy(p)

    if not args.no_cpu:
        import oracle
        Hh, Gh = H.cpu().numpy(), G.cpu().numpy()
        def cpu_step(threads):
            t0 = time.perf_counter()
            oracle.spmm(g.rowptr, g.colidx, g.vals, Hh, want_abs=False, threads=threads)
            oracle.spmm_t(g.rowptr, g.colidx, g.vals, Gh, want_abs=False, threads=threads)
            return time.perf_counter() - t0
        multi = sorted(cpu_step(True) for _ in range(3))[1]
        single = cpu_step(False)
        out["cpu_baseline"] = {"value": round(flop / multi / 1e9, 3), "unit": "GFLOP/s",
                               "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": f"the same workload, whole steps (1 forward + 1 backward aggregation): median of 3 "
                                         f"steps with OpenMP ({multi:.2f} s each) and 1 step single-threaded ({single:.2f} s), fp64",
                               "single_thread_value": round(flop / single / 1e9, 3)}
        log(f"[bench] cpu oracle: {multi:.2f}s with {oracle.num_threads()} threads, {single:.2f}s single-threaded")
    ag.ag_plan_destroy(plan)
    del H, G, Hp, Gp, Y, dH
    torch.cuda.empty_cache()
    if not args.no_mixed:
        out["adaptive_vs_single_format"] = adaptive_vs_single_format(4, max(50, args.steps))
    if args.all_configs:
        out["other_workloads"] = [brief(i, max(50, args.steps)) for i in range(len(CONFIGS)) if i != args.config]
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
