#!/usr/bin/env python3
"""Benchmark of the pLogP tuning sweep on one MI355X.

A step is one pass of the whole hot path (table terms, Scatter sums, sweep
over s, arg-min over strategies, decision-table write: one plogp_tune_grid
call) over one synthetic workload whose tables and grid are already resident
in HBM.  The headline workload is config 2; configs 3-5 are timed too and
reported under "workloads" in the same JSON line.  Beside the step, per
workload: the same call replayed from a HIP graph, the cut-over extraction of
the table just tuned, the scoring of predictions against synthetic
measurements and (batches) the robustness summary, each with its own roofline
and the oracle timed on the host.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--extra 3,4,5] [--no-cpu]
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

METRIC = "pLogP model evaluations/sec (strategy×m×P×s) + decision-table cells/sec"
FP64_VECTOR_PEAK = 78.6e12        # flop/s: 256 CU x 4 SIMD x 16 lanes x 2 flop x 2.4 GHz
HBM_PEAK = 8.0e12                 # bytes/s
STAGES = ("terms", "chain_blocks", "chain_prefix", "sweep")

# flops of one unsegmented row per (m, P), arg-min compare included
# (convention: fma = 2, add/mul/compare = 1, select/convert/integer = 0)
UNSEG_FLOPS = {0: 3, 1: 3, 3: 3, 4: 3, 6: 4, 7: 4, 8: 4, 10: 3, 11: 4, 12: 3}


def algorithmic_work(wl):
    """Flops and bytes the method itself needs per stage (after hoisting the
    terms of the segmented rows that do not depend on P), per tune call."""
    c = wl.counts()
    mask, nt, n = wl.strategy_mask, wl.n_tables, wl.sizes.shape[1]
    n_m, n_P, n_s = len(wl.m), len(wl.P), len(wl.s)
    Pmax = int(wl.P.max())
    cl_max = (Pmax - 1).bit_length()
    search = math.ceil(math.log2(n))
    interp = search + 3                                   # compares + sub + fma
    n_seg = sum(1 for i in (2, 5, 9) if (mask >> i) & 1)
    seg_evals = c["ms_pairs"] * n_P * n_seg
    unseg = sum(f for i, f in UNSEG_FLOPS.items() if (mask >> i) & 1)
    work = {
        "terms": {"flops": nt * ((n - 1) * 3 + interp * (1 + n_s + n_m * (1 + (cl_max if (mask >> 12) & 1 else 0)))),
                  "bytes": nt * n * 16},
        "chain_blocks": {"flops": 6 * c["scatter_chain_interps"], "bytes": 0},
        "chain_prefix": {"flops": nt * n_m * ((Pmax - 1) // 64) if (mask >> 11) & 1 else 0, "bytes": 0},
        "sweep": {"flops": 3 * seg_evals + 5 * c["ms_pairs"] + unseg * nt * n_m * n_P,
                  "bytes": c["output_bytes"]},
    }
    return work, c


def describe(wl):
    return "%s: %d table(s) x %d samples, %d m x %d P x %d s, mask 0x%x" % (
        wl.name, wl.n_tables, wl.sizes.shape[1], len(wl.m), len(wl.P), len(wl.s), wl.strategy_mask)


# HBM bytes per launch (fetched + written) of each stage's kernel, from rocprofv3 --pmc
# FETCH_SIZE / WRITE_SIZE runs of this file, scaled by what the same counters read for a copy
# kernel of known size (profiles/tune_grid_cfg<N>_kernel_stats.txt, section 2).
MEASURED_TRAFFIC = {
    2: {"sweep": 0.336e6 + 33.560e6},
    3: {"chain_blocks": 0.387e6 + 1.496e6, "sweep": 4.016e6 + 2.294e6},
    4: {"terms": 5.283e6 + 10.736e6, "sweep": 88.979e6 + 1966.079e6},
    5: {"chain_blocks": 1.839e6 + 73.536e6,
        "chain_prefix": 50.976e6 + 18.581e6, "sweep": 44.802e6 + 93.321e6},
}
# the same for the kernels of the cut-over extraction (mark, scan1 [+ scan2 on config 4], emit)
MEASURED_CUT_TRAFFIC = {
    2: 34.270e6 + 2.095e6 + 0.563e6 + 0.526e6 + 9.296e6 + 0.486e6,
    3: 2.387e6 + 0.141e6 + 0.060e6 + 0.035e6 + 1.734e6 + 0.982e6,
    4: 1993.133e6 + 61.704e6 + 30.754e6 + 30.840e6 + 0.035e6 + 0.030e6 + 297.974e6 + 52.548e6,
    5: 97.012e6 + 5.952e6 + 1.497e6 + 1.464e6 + 26.717e6 + 0.865e6,
}
# the scoring kernels (k_score, k_score_rows, k_score_final) and the robustness summary
# (k_robust_clear, k_robust; its per-table counts are one atomic per wave and table, which the
# write counter sees as 86 MB)
MEASURED_SCORE_TRAFFIC = {
    2: 139.182e6 + 144.107e6 + 221.466e6 + 0.213e6 + 0.256e6,
    3: 11.925e6 + 9.961e6 + 14.767e6 + 0.213e6 + 0.256e6,
    4: 1.516e6 + 0.836e6 + 1.350e6 + 0.053e6 + 0.096e6,
    5: 401.050e6 + 400.357e6 + 623.124e6 + 0.852e6 + 0.895e6,
}
MEASURED_ROBUST_TRAFFIC = {4: 0.021e6 + 0.187e6 + 1967.171e6 + 86.391e6}


def roofline_of(stage, work, ms, traffic=None):
    r = _roofline_of(stage, work, ms)
    r["traffic"] = traffic
    return r


def _roofline_of(stage, work, ms):
    w = work[stage]
    t_alu = w["flops"] / FP64_VECTOR_PEAK
    t_hbm = w["bytes"] / HBM_PEAK
    sec = ms * 1e-3
    if t_hbm > t_alu:
        ach = w["bytes"] / sec / 1e9
        return {"kernel": stage, "bound": "hbm", "achieved": ach, "peak": HBM_PEAK / 1e9,
                "unit": "GB/s", "frac": ach / (HBM_PEAK / 1e9), "traffic": None,
                "algorithmic_bytes": w["bytes"], "avg_ms": ms}
    ach = w["flops"] / sec / 1e12
    return {"kernel": stage, "bound": "alu", "achieved": ach, "peak": FP64_VECTOR_PEAK / 1e12,
            "unit": "TFLOP/s", "frac": ach / (FP64_VECTOR_PEAK / 1e12), "traffic": None,
            "algorithmic_flops": w["flops"], "avg_ms": ms}


def run_gpu(wl, steps, warmup, profile_reps, with_cut=True):
    import torch
    from paper_cs_0408034_amd import plogp

    torch.cuda.set_device(0)
    tab = plogp.plogp_load_tables(wl.sizes, wl.gaps, wl.L)
    grid = plogp.plogp_grid_create(wl.m, wl.P, wl.s, wl.s_cap, wl.dtype_size, wl.strategy_mask)
    nbytes = plogp.plogp_decision_table_bytes(tab.count, grid)
    out = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()
    sh = stream.cuda_stream
    for _ in range(warmup):
        plogp.plogp_tune_grid(tab, grid, out.data_ptr(), nbytes, sh)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(steps):
        plogp.plogp_tune_grid(tab, grid, out.data_ptr(), nbytes, sh)
    e1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ev_ms = e0.elapsed_time(e1)
    ms_per_step = max(wall_ms, ev_ms) / steps
    # the same call captured once in a HIP graph and replayed (what a caller with a launch-bound
    # loop would do); reported beside the eager figure, never as `value`
    graph_ms = None
    if with_cut:
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            plogp.plogp_tune_grid(tab, grid, out.data_ptr(), nbytes, side.cuda_stream)
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            plogp.plogp_tune_grid(tab, grid, out.data_ptr(), nbytes, torch.cuda.current_stream().cuda_stream)
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        g0.record(stream)
        for _ in range(steps):
            graph.replay()
        g1.record(stream)
        torch.cuda.synchronize()
        graph_ms = max((time.perf_counter() - t0) * 1e3, g0.elapsed_time(g1)) / steps
        del graph
    # per-kernel durations: every kernel launched profile_reps times back to back between two
    # HIP events on the launch stream; the median of five such rounds
    rounds = [plogp.plogp_tune_grid_profile(tab, grid, out.data_ptr(), nbytes, sh, profile_reps)
              for _ in range(5)]
    stage_ms = dict(zip(STAGES, np.median(np.array(rounds), axis=0).tolist()))
    cut = run_cutovers(plogp, torch, wl, tab, grid, out, nbytes, stream, steps, profile_reps) if with_cut else None
    if cut is not None and wl.name in ("cfg2", "cfg3", "cfg4", "cfg5") and wl.counts()["cells"] == nbytes // 16:
        cut["roofline"]["traffic"] = MEASURED_CUT_TRAFFIC.get(int(wl.name[3:]))
    score = run_score(plogp, torch, wl, tab, grid, stream, steps, profile_reps) if with_cut else None
    full = wl.name in ("cfg2", "cfg3", "cfg4", "cfg5") and wl.counts()["cells"] == nbytes // 16
    if score is not None and full and wl.strategy_mask == 0x1FFF:
        score["roofline"]["traffic"] = MEASURED_SCORE_TRAFFIC.get(int(wl.name[3:]))
    if score is not None and tab.count > 1:
        score["robustness"] = run_robustness(plogp, torch, tab, grid, out, nbytes, stream, steps,
                                             profile_reps)
        if full:
            score["robustness"]["roofline"]["traffic"] = MEASURED_ROBUST_TRAFFIC.get(int(wl.name[3:]))
    del out
    grid.free()
    tab.free()
    return ms_per_step, stage_ms, cut, score, graph_ms


CUT_STAGES = ("mark", "scan", "emit")
SCORE_STAGES = ("terms", "score", "statistics")


def run_score(plogp, torch, wl, tab, grid, stream, steps, profile_reps):
    """Prediction against measurement for table 0 of the workload on its (m, P) grid:
    synthetic measured times of every enabled strategy, already resident."""
    from plogp_workloads import make_measurements
    sh = stream.cuda_stream
    meas, seg = make_measurements(wl)
    rows, n_m, n_P = meas.shape
    assert rows == plogp.plogp_score_strategies(grid)
    d_meas = torch.from_numpy(meas).cuda()
    d_seg = torch.from_numpy(seg.view(np.int32)).cuda()
    d_pred = torch.empty_like(d_meas)
    d_ver = torch.empty(grid.ops * n_m * n_P * 16, dtype=torch.uint8, device="cuda")
    d_sc = torch.empty(rows * 32, dtype=torch.uint8, device="cuda")
    args = (tab, 0, grid, d_meas.data_ptr(), d_seg.data_ptr(), d_pred.data_ptr(), d_ver.data_ptr(),
            d_sc.data_ptr(), sh)
    for _ in range(3):
        plogp.plogp_score_grid(*args)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(steps):
        plogp.plogp_score_grid(*args)
    e1.record(stream)
    torch.cuda.synchronize()
    ms = max((time.perf_counter() - t0) * 1e3, e0.elapsed_time(e1)) / steps
    rounds = [plogp.plogp_score_grid_profile(*args, profile_reps) for _ in range(5)]
    stage_ms = dict(zip(SCORE_STAGES, np.median(np.array(rounds), axis=0).tolist()))
    # what the scoring has to move: every measured time read once, the segment size of the
    # segmented strategies' points, every prediction and every verdict written once (the
    # statistics could in principle be formed from values already in registers)
    points = n_m * n_P
    n_seg = sum(1 for i in (2, 5, 9) if (wl.strategy_mask >> i) & 1)
    alg_bytes = points * (8 * rows + 4 * n_seg + 8 * rows + 16 * grid.ops) + 32 * rows
    k_ms = stage_ms["score"] + stage_ms["statistics"]
    ach = alg_bytes / (k_ms * 1e-3) / 1e9
    return {"ms_per_call": ms, "points_per_s": rows * points / (ms * 1e-3), "strategies": rows,
            "points": points, "stage_ms": stage_ms,
            "roofline": {"kernel": "score+statistics", "bound": "hbm", "achieved": ach,
                         "peak": HBM_PEAK / 1e9, "unit": "GB/s", "frac": ach / (HBM_PEAK / 1e9),
                         "traffic": None, "algorithmic_bytes": alg_bytes, "avg_ms": k_ms}}


def run_robustness(plogp, torch, tab, grid, out, nbytes, stream, steps, profile_reps):
    """The robustness summary over the batch just tuned (table 0 against all the others)."""
    sh = stream.cuda_stream
    nt = tab.count
    per_table = nbytes // 16 // nt
    d_agree = torch.empty(per_table, dtype=torch.int32, device="cuda")
    d_dev = torch.empty(per_table, dtype=torch.float64, device="cuda")
    d_tab = torch.empty(nt, dtype=torch.int32, device="cuda")
    args = (grid, nt, out.data_ptr(), plogp.KEY_STRATEGY_AND_SEGMENT, d_agree.data_ptr(),
            d_dev.data_ptr(), d_tab.data_ptr(), sh)
    for _ in range(3):
        plogp.plogp_robustness(*args)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(steps):
        plogp.plogp_robustness(*args)
    e1.record(stream)
    torch.cuda.synchronize()
    ms = max((time.perf_counter() - t0) * 1e3, e0.elapsed_time(e1)) / steps
    k_ms = float(np.median([plogp.plogp_robustness_profile(*args, profile_reps) for _ in range(5)]))
    # every 16-byte record of every table read once; 12 bytes per cell position and 4 per table out
    alg_bytes = nbytes + 12 * per_table + 4 * nt
    ach = alg_bytes / (k_ms * 1e-3) / 1e9
    return {"ms_per_call": ms, "cells_per_s": (nbytes // 16) / (ms * 1e-3), "tables": nt,
            "mean_fraction_kept": float(d_agree.double().mean().item()) / max(nt - 1, 1),
            "roofline": {"kernel": "k_robust", "bound": "hbm", "achieved": ach, "peak": HBM_PEAK / 1e9,
                         "unit": "GB/s", "frac": ach / (HBM_PEAK / 1e9), "traffic": None,
                         "algorithmic_bytes": alg_bytes, "avg_ms": k_ms}}


def robust_cpu(sample):
    """The robustness oracle (array operations, one thread) on the oracle's tables of the sample."""
    import oracle
    from oracle import plogp_robust as orb
    cells, _ = oracle.tune_workload(sample)
    runs, dt = 0, 0.0
    while dt < 1.0 and runs < 20:
        t0 = time.perf_counter()
        orb.robustness(cells, 1)
        dt += time.perf_counter() - t0
        runs += 1
    return {"value": runs * cells.size / dt, "unit": "cells/s", "cores": 1, "kind": "oracle",
            "seconds": dt}


def score_cpu(sample):
    """The scoring oracle (one thread) on table 0 of the sample; a big table with long chain sums
    (config 5) is cut down further to every 16th of the sample's sizes (a few seconds of work)."""
    import dataclasses
    import oracle
    from plogp_workloads import make_measurements
    if sample.sizes.shape[1] > 1024 and len(sample.m) > 64:
        sample = dataclasses.replace(sample, m=sample.m[::16])
    meas, seg = make_measurements(sample)
    a = (sample.sizes[0], sample.gaps[0], float(sample.L[0]), sample.m, sample.P, sample.strategy_mask,
         meas, seg)
    runs, dt = 0, 0.0
    while dt < 1.0 and runs < 20:
        t0 = time.perf_counter()
        oracle.score_grid(*a)
        dt += time.perf_counter() - t0
        runs += 1
    return {"value": runs * meas.size / dt, "unit": "points/s", "cores": 1, "kind": "oracle",
            "seconds": dt}


def run_cutovers(plogp, torch, wl, tab, grid, out, nbytes, stream, steps, profile_reps):
    """The cut-over extraction (runs of equal (strategy, s) along m) of the table just tuned."""
    sh = stream.cuda_stream
    n_cells = nbytes // 16
    rows = plogp.plogp_cutover_rows(tab.count, grid)
    d_off = torch.empty(rows + 1, dtype=torch.int64, device="cuda")
    cap = n_cells                      # one record per cell always suffices
    d_runs = torch.empty(cap * 16, dtype=torch.uint8, device="cuda")
    args = (grid, tab.count, out.data_ptr(), plogp.KEY_STRATEGY_AND_SEGMENT, d_off.data_ptr(),
            d_runs.data_ptr(), cap, sh)
    for _ in range(3):
        plogp.plogp_cutovers(*args)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(steps):
        plogp.plogp_cutovers(*args)
    e1.record(stream)
    torch.cuda.synchronize()
    ms = max((time.perf_counter() - t0) * 1e3, e0.elapsed_time(e1)) / steps
    n_runs = int(d_off[-1].item())
    assert n_runs <= cap, "bench: run buffer too small (%d runs)" % n_runs
    rounds = [plogp.plogp_cutovers_profile(*args, profile_reps) for _ in range(5)]
    stage_ms = dict(zip(CUT_STAGES, np.median(np.array(rounds), axis=0).tolist()))
    # what the extraction itself has to move: the 8-byte key of every cell once, a 16-byte
    # record per run, an 8-byte offset per row
    alg_bytes = 8 * n_cells + 16 * n_runs + 8 * (rows + 1)
    kernels_ms = sum(stage_ms.values())
    ach = alg_bytes / (kernels_ms * 1e-3) / 1e9
    return {"ms_per_call": ms, "cells_per_s": n_cells / (ms * 1e-3), "runs": n_runs, "rows": rows,
            "key": "strategy and segment size", "stage_ms": stage_ms,
            "roofline": {"kernel": "mark+scan+emit", "bound": "hbm", "achieved": ach,
                         "peak": HBM_PEAK / 1e9, "unit": "GB/s", "frac": ach / (HBM_PEAK / 1e9),
                         "traffic": None, "algorithmic_bytes": alg_bytes, "avg_ms": kernels_ms}}


def cut_cpu(sample):
    """The oracle's extraction (array operations, one thread) on the oracle's table of the sample."""
    import oracle
    from oracle import plogp_cutover as oc
    cells, _ = oracle.tune_workload(sample)
    oc.cutovers(cells[:1, :, :, :2], sample.m, 1)
    runs, dt = 0, 0.0
    while dt < 1.0 and runs < 20:
        t0 = time.perf_counter()
        oc.cutovers(cells, sample.m, 1)
        dt += time.perf_counter() - t0
        runs += 1
    return {"value": runs * cells.size / dt, "unit": "cells/s", "cores": 1, "kind": "oracle",
            "seconds": dt}


def cpu_sample(cfg, wl):
    """A bounded cut of the same workload for the oracle (a few seconds of work)."""
    from plogp_workloads import make_workload
    if cfg == 3:
        return make_workload(3, m_slice=slice(0, 1024, 8)), "every 8th m row of config 3 (128 of 1024), all P, all s"
    if cfg == 4:
        return make_workload(4, n_tables=100), "first 100 of the 10 000 tables of config 4, full grid"
    if cfg == 5:
        return make_workload(5, m_slice=slice(0, 4096, 8)), "every 8th m row of config 5 (512 of 4096), all P, all s"
    return wl, "the full %s workload" % wl.name


def run_cpu(cfg, wl):
    import oracle
    sample, what = cpu_sample(cfg, wl)
    oracle.tune_grid(sample.sizes[:1], sample.gaps[:1], sample.L[:1], sample.m[:2], sample.P[:2],
                     sample.s, sample.s_cap, sample.strategy_mask)          # load + warm
    runs, dt = 0, 0.0
    while dt < 1.5 and runs < 50:               # about 1.5 s of wall time on all cores
        t0 = time.perf_counter()
        _, used = oracle.tune_workload(sample)
        dt += time.perf_counter() - t0
        runs += 1
    c = sample.counts()
    return {"value": runs * c["nominal_evals"] / dt, "unit": "evaluations/s", "cores": int(used),
            "kind": "oracle", "sample": "%s, %d run(s)" % (what, runs), "seconds": dt,
            "effective_evals_per_s": runs * c["effective_evals"] / dt,
            "cells_per_s": runs * c["cells"] / dt}


def bench_config(cfg, steps, warmup, with_cpu, mask=None):
    from plogp_workloads import make_workload
    wl = make_workload(cfg)
    if mask is not None:
        wl.strategy_mask = mask
    work, c = algorithmic_work(wl)
    ms, stage_ms, cut, score, graph_ms = run_gpu(wl, steps, warmup, profile_reps=max(5, min(steps, 20)))
    traffic = MEASURED_TRAFFIC.get(cfg, {}) if mask is None else {}
    if stage_ms["terms"] == 0.0 and stage_ms["sweep"] > 0.0:
        # the single-kernel batch path did every stage inside one launch
        work = {"terms": {"flops": 0, "bytes": 0}, "chain_blocks": {"flops": 0, "bytes": 0},
                "chain_prefix": {"flops": 0, "bytes": 0},
                "sweep": {"flops": sum(w["flops"] for w in work.values()),
                          "bytes": sum(w["bytes"] for w in work.values())}}
    elif stage_ms["terms"] < 0.001 < stage_ms["chain_blocks"]:
        # the terms and the chain sums run in one launch (side by side for small tables, the
        # terms at the end of each workgroup for big ones), timed under "chain_blocks"
        work = dict(work)
        work["chain_blocks"] = {k: work["chain_blocks"][k] + work["terms"][k] for k in ("flops", "bytes")}
        work["terms"] = {"flops": 0, "bytes": 0}
    dominant = max(STAGES, key=lambda k: stage_ms[k])
    res = {
        "workload": describe(wl),
        "ms_per_step": ms,
        "value": c["nominal_evals"] / (ms * 1e-3),
        "effective_evals_per_s": c["effective_evals"] / (ms * 1e-3),
        "cells_per_s": c["cells"] / (ms * 1e-3),
        "scatter_chain_interps_per_s": c["scatter_chain_interps"] / (ms * 1e-3),
        "steps": steps,
        "graph_replay_ms_per_step": graph_ms,
        "stage_ms": stage_ms,
        "roofline": roofline_of(dominant, work, stage_ms[dominant], traffic.get(dominant)),
        "stage_rooflines": {k: roofline_of(k, work, stage_ms[k], traffic.get(k))
                            for k in STAGES if stage_ms[k] > 0},
    }
    if cut is not None:
        res["cutover_extraction"] = cut
    if score is not None:
        res["prediction_scoring"] = score
    if with_cpu:
        res["cpu_baseline"] = run_cpu(cfg, wl)
        if cut is not None:
            sample, what = cpu_sample(cfg, wl)
            cut["cpu_baseline"] = dict(cut_cpu(sample), sample=what)
        if score is not None:
            sample, what = cpu_sample(cfg, wl)
            thin = ", every 16th size of it" if sample.sizes.shape[1] > 1024 and len(sample.m) > 64 else ""
            score["cpu_baseline"] = dict(score_cpu(sample), sample="table 0 of: " + what + thin)
            if "robustness" in score:
                score["robustness"]["cpu_baseline"] = dict(robust_cpu(sample), sample=what)
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2, help="headline workload (1..5)")
    ap.add_argument("--extra", type=str, default="3,4,5", help="other configs to time, or 'none'")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--mask", type=lambda v: int(v, 0), default=None,
                    help="strategy mask override (for profiling parts of the path)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one elementwise kernel that copies 256 MiB (known traffic, "
                         "to scale the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no inter-GPU path exists); use --gpus 1")

    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the library has no CPU fallback")

    if args.calibrate_copy:
        # One elementwise kernel that reads 256 MiB and writes 256 MiB (float64 add of 0):
        # the plain copy of known size that the HBM counters are scaled by.
        a = torch.ones(32 << 20, dtype=torch.float64, device="cuda")
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        torch.add(a, 0.0, out=b)
        torch.cuda.synchronize()
        del a, b
    head = bench_config(args.config, args.steps, args.warmup, not args.no_cpu, args.mask)
    line = {
        "metric": METRIC,
        "value": head["value"],
        "unit": "evaluations/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f64",
        "data": "synthetic",
        "config": {"workload": head["workload"]},
        "cells_per_s": head["cells_per_s"],
        "effective_evals_per_s": head["effective_evals_per_s"],
        "graph_replay_ms_per_step": head["graph_replay_ms_per_step"],
        "stage_ms": head["stage_ms"],
        "roofline": head["roofline"],
        "stage_rooflines": head["stage_rooflines"],
    }
    if "cpu_baseline" in head:
        line["cpu_baseline"] = head["cpu_baseline"]
    if "cutover_extraction" in head:
        line["cutover_extraction"] = head["cutover_extraction"]
    if "prediction_scoring" in head:
        line["prediction_scoring"] = head["prediction_scoring"]
    extras = [] if args.extra in ("", "none") else [int(v) for v in args.extra.split(",")]
    if extras:
        line["workloads"] = {}
        for cfg in extras:
            if cfg == args.config:
                continue
            # enough steps and warm-up for the clocks to settle (50 steps read 10 % slow)
            line["workloads"]["cfg%d" % cfg] = bench_config(cfg, 300, 20, not args.no_cpu)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
