#!/usr/bin/env python3
"""Benchmark of the pLogP tuning sweep on one MI355X.

A step is one pass of the whole hot path (table terms, Scatter sums, sweep
over s, arg-min over strategies, decision-table write: one plogp_tune_grid
call) over one synthetic workload whose tables and grid are already resident
in HBM.  The headline workload is config 4 (10 000 tables: the largest job
that one GPU holds); configs 3, 5 and 2 are timed the same way and reported,
shortened, under "workloads"; the steps after the sweep (cut-over extraction,
prediction scoring, robustness summary) under "next".

Timing: whatever --steps says, a call is timed as the median of at least five
batches of at least 100 back-to-back calls between two HIP events on the
launch stream; per-kernel times are the median of five rounds in which every
kernel of the call is launched 100 times between two events
(plogp_*_profile).  The published peaks a fraction is taken of stand beside
what a bare multiply-add kernel and a bare fill kernel reach on this device
in the same run ("measured_ceiling").

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--extra 3,5,2] [--no-cpu]
                    [--no-next] [--detail FILE]
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
VALU_ISSUE_PEAK = 39.3e12         # lane-instructions/s: 256 CU x 4 SIMD x 16 lanes x 2.4 GHz
HBM_PEAK = 8.0e12                 # bytes/s
STAGES = ("terms", "chain_blocks", "chain_prefix", "sweep", "more_planes")
MIN_BATCHES, MIN_PER_BATCH = 5, 100

# flops of one unsegmented row per (m, P), arg-min compare included
# (convention: fma = 2, add/mul/compare = 1, select/convert/integer = 0)
UNSEG_FLOPS = {0: 3, 1: 3, 3: 3, 4: 3, 6: 4, 7: 4, 8: 4, 10: 3, 11: 4, 12: 3}

# Counter readings of the dominant kernel of each config, taken OFFLINE by rocprofv3 --pmc runs
# of this file (summaries, with their commands, in profiles/tune_grid_cfg<N>_kernel_stats.txt)
# - not measured in this run: HBM bytes per launch (FETCH_SIZE + WRITE_SIZE, each scaled by what
# the same counter reads for a copy of known size) and vector instructions issued per launch
# (SQ_INSTS_VALU, in wave instructions).  A kernel change makes them stale until the profiles
# are taken again; the line names its source.
OFFLINE_COUNTERS = {
    2: {"kernel": "k_row", "hbm_bytes": 0.336e6 + 34.317e6, "valu_insts": 4.864e6},
    3: {"kernel": "k_sweep_s", "hbm_bytes": 4.022e6 + 2.681e6, "valu_insts": 33.84e6},
    4: {"kernel": "k_batch_t", "hbm_bytes": 87.199e6 + 1966.357e6, "valu_insts": 175.7e6},
    5: {"kernel": "k_chain_blocks", "hbm_bytes": 1.840e6 + 73.784e6, "valu_insts": 25.60e6},
}


def algorithmic_work(wl):
    """Per stage and per tune call: the flops and bytes the method delivers ("delivered": 3 flop
    per segmented value for each of the three segmented rows, 6 flop per Scatter-chain term for
    every grid m, repeats included) and the ones the kernels have to execute after the exact
    shortcuts ("executed": rows 2 and 9 of Table 1 through min_s A, one min per (m, s); the
    chain sums once per distinct m)."""
    c = wl.counts()
    mask, nt, n = wl.strategy_mask, wl.n_tables, wl.sizes.shape[1]
    n_m, n_P, n_s = len(wl.m), len(wl.P), len(wl.s)
    n_mu = len(np.unique(wl.m))
    Pmax = int(wl.P.max())
    cl_max = (Pmax - 1).bit_length()
    interp = math.ceil(math.log2(n)) + 3                  # compares + sub + fma
    n_seg = sum(1 for i in (2, 5, 9) if (mask >> i) & 1)
    pairs = c["ms_pairs"]
    unseg = sum(f for i, f in UNSEG_FLOPS.items() if (mask >> i) & 1)
    terms = nt * ((n - 1) * 3 + interp * (1 + n_s + n_m * (1 + (cl_max if (mask >> 12) & 1 else 0))))
    chain = 6 * c["scatter_chain_interps"]
    chain_x = chain * n_mu // n_m
    prefix = nt * n_m * ((Pmax - 1) // 64) if (mask >> 11) & 1 else 0
    sweep = 3 * pairs * n_P * n_seg + 5 * pairs + unseg * nt * n_m * n_P
    seg5 = 1 if (mask >> 5) & 1 else 0
    sweep_x = 3 * pairs * n_P * seg5 + (pairs if mask & 0x204 else 0) + 5 * pairs + unseg * nt * n_m * n_P
    # the planes of Gather and Barrier (rows beyond the tables; none in the five configs)
    planes = [bool(mask & b) for b in (0x3FF, 0x1C00, 0xE000, 0x30000)]
    more_bytes = c["output_bytes"] * sum(planes[2:]) // max(sum(planes), 1)
    more_flops = nt * n_m * n_P * (sum(UNSEG_FLOPS[i - 3] for i in (13, 14, 15) if (mask >> i) & 1) +
                                   sum(4 for i in (16, 17) if (mask >> i) & 1))
    return {
        "terms": {"flops": terms, "flops_executed": terms, "bytes": nt * n * 16},
        "chain_blocks": {"flops": chain, "flops_executed": chain_x, "bytes": 0},
        "chain_prefix": {"flops": prefix, "flops_executed": prefix * n_mu // n_m, "bytes": 0},
        "sweep": {"flops": sweep, "flops_executed": sweep_x, "bytes": c["output_bytes"] - more_bytes},
        "more_planes": {"flops": more_flops, "flops_executed": more_flops, "bytes": more_bytes},
    }, c


def describe(wl):
    return "%s: %d table(s) x %d samples, %d m x %d P x %d s, mask 0x%x" % (
        wl.name, wl.n_tables, wl.sizes.shape[1], len(wl.m), len(wl.P), len(wl.s), wl.strategy_mask)


def roofline_of(stage, work, ms, ceilings=None, offline=None):
    """The roofline object of one kernel: bound by whichever of its algorithmic flop time and
    byte time is larger; achieved = delivered work per launch / average launch duration."""
    w = work[stage]
    sec = ms * 1e-3
    r4 = lambda v: float("%.4g" % v)
    if w["bytes"] / HBM_PEAK > w["flops"] / FP64_VECTOR_PEAK:
        ach = w["bytes"] / sec / 1e9
        r = {"kernel": stage, "bound": "hbm", "achieved": r4(ach), "peak": HBM_PEAK / 1e9, "unit": "GB/s",
             "frac": r4(ach / (HBM_PEAK / 1e9)), "traffic": None, "algorithmic_bytes": w["bytes"], "avg_ms": r4(ms)}
        if ceilings:
            r["measured_ceiling"] = r4(ceilings["store_gbs"])
            r["frac_of_measured_ceiling"] = r4(ach / ceilings["store_gbs"])
    else:
        ach = w["flops"] / sec / 1e12
        r = {"kernel": stage, "bound": "alu", "achieved": r4(ach), "peak": FP64_VECTOR_PEAK / 1e12,
             "unit": "TFLOP/s", "frac": r4(ach / (FP64_VECTOR_PEAK / 1e12)), "traffic": None,
             "frac_executed": r4(w["flops_executed"] / sec / FP64_VECTOR_PEAK),
             "algorithmic_flops": w["flops"], "executed_flops": w["flops_executed"], "avg_ms": r4(ms)}
        if ceilings:
            r["measured_ceiling"] = r4(ceilings["fma_tflops"])
    r["frac_delivered"] = r["frac"]
    if offline:
        r["kernel"] = "%s (%s)" % (stage, offline["kernel"])
        r["traffic"] = offline["hbm_bytes"]
        r["counters_source"] = "offline rocprofv3 --pmc, profiles/tune_grid_cfg%d_kernel_stats.txt" % offline["cfg"]
        if offline.get("valu_insts"):
            r["valu_issue_util"] = r4(offline["valu_insts"] * 64 / (VALU_ISSUE_PEAK * sec))
    return r


def timed_calls(torch, stream, call, steps, warmup):
    """Median milliseconds per call over at least MIN_BATCHES batches of at least MIN_PER_BATCH
    calls, each batch between two events on `stream` (and never less than the host saw)."""
    per_batch = max(MIN_PER_BATCH, steps)
    for _ in range(max(warmup, 3)):
        call()
    torch.cuda.synchronize()
    times = []
    for _ in range(MIN_BATCHES):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record(stream)
        for _ in range(per_batch):
            call()
        e1.record(stream)
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        times.append(max(wall_ms, e0.elapsed_time(e1)) / per_batch)
    return float(np.median(times)), per_batch


def run_gpu(wl, steps, warmup, with_next, ceilings_wanted):
    import torch
    from paper_cs_0408034_amd import plogp

    torch.cuda.set_device(0)
    tab = plogp.plogp_load_tables(wl.sizes, wl.gaps, wl.L)
    grid = plogp.plogp_grid_create(wl.m, wl.P, wl.s, wl.s_cap, wl.dtype_size, wl.strategy_mask)
    nbytes = plogp.plogp_decision_table_bytes(tab.count, grid)
    out = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()
    sh = stream.cuda_stream
    ms, per_batch = timed_calls(torch, stream,
                                lambda: plogp.plogp_tune_grid(tab, grid, out.data_ptr(), nbytes, sh), steps, warmup)
    # per-kernel durations: every kernel launched MIN_PER_BATCH times back to back between two HIP
    # events on the launch stream; the median of five such rounds
    rounds = [plogp.plogp_tune_grid_profile(tab, grid, out.data_ptr(), nbytes, sh, MIN_PER_BATCH)
              for _ in range(MIN_BATCHES)]
    stage_ms = dict(zip(STAGES, np.median(np.array(rounds), axis=0).tolist()))
    res = {"ms": ms, "per_batch": per_batch, "stage_ms": stage_ms}
    if ceilings_wanted:
        side = torch.empty(max(nbytes, 1 << 30), dtype=torch.uint8, device="cuda")
        fma, store = plogp.plogp_measure_ceilings(side.data_ptr(), side.numel(), sh)
        res["ceilings"] = {"fma_tflops": fma, "store_gbs": store}
        del side
        plogp.plogp_tune_grid(tab, grid, out.data_ptr(), nbytes, sh)
    if with_next:
        res["cutovers"] = run_cutovers(plogp, torch, wl, tab, grid, out, nbytes, stream, steps)
        res["scoring"] = run_score(plogp, torch, wl, tab, grid, stream, steps)
        if tab.count > 1:
            res["robustness"] = run_robustness(plogp, torch, tab, grid, out, nbytes, stream, steps)
    del out
    grid.free()
    tab.free()
    return res


def hbm_leg(ms, k_ms, alg_bytes, extra):
    ach = alg_bytes / (k_ms * 1e-3) / 1e9
    r = {"ms_per_call": float("%.4g" % ms), "kernels_ms": float("%.4g" % k_ms),
         "roofline": {"bound": "hbm", "achieved": float("%.4g" % ach), "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                      "frac": float("%.3g" % (ach / (HBM_PEAK / 1e9))), "algorithmic_bytes": alg_bytes}}
    r.update(extra)
    return r


def run_score(plogp, torch, wl, tab, grid, stream, steps):
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
    ms, _ = timed_calls(torch, stream, lambda: plogp.plogp_score_grid(*args), steps, 3)
    rounds = [plogp.plogp_score_grid_profile(*args, MIN_PER_BATCH) for _ in range(MIN_BATCHES)]
    st = np.median(np.array(rounds), axis=0).tolist()
    # what the scoring has to move: every measured time read once, the segment size of the
    # segmented strategies' points, every prediction and every verdict written once
    points = n_m * n_P
    n_seg = sum(1 for i in (2, 5, 9) if (wl.strategy_mask >> i) & 1)
    alg_bytes = points * (8 * rows + 4 * n_seg + 8 * rows + 16 * grid.ops) + 32 * rows
    return hbm_leg(ms, st[1] + st[2], alg_bytes,
                   {"points_per_s": float("%.4g" % (rows * points / (ms * 1e-3))),
                    "stage_ms": {"terms": st[0], "score": st[1], "statistics": st[2]}})


def run_robustness(plogp, torch, tab, grid, out, nbytes, stream, steps):
    """The robustness summary over the batch just tuned (table 0 against all the others)."""
    sh = stream.cuda_stream
    nt = tab.count
    per_table = nbytes // 16 // nt
    d_agree = torch.empty(per_table, dtype=torch.int32, device="cuda")
    d_dev = torch.empty(per_table, dtype=torch.float64, device="cuda")
    d_tab = torch.empty(nt, dtype=torch.int32, device="cuda")
    args = (grid, nt, out.data_ptr(), plogp.KEY_STRATEGY_AND_SEGMENT, d_agree.data_ptr(),
            d_dev.data_ptr(), d_tab.data_ptr(), sh)
    ms, _ = timed_calls(torch, stream, lambda: plogp.plogp_robustness(*args), steps, 3)
    k_ms = float(np.median([plogp.plogp_robustness_profile(*args, MIN_PER_BATCH) for _ in range(MIN_BATCHES)]))
    # every 16-byte record of every table read once; 12 bytes per cell position and 4 per table out
    alg_bytes = nbytes + 12 * per_table + 4 * nt
    return hbm_leg(ms, k_ms, alg_bytes,
                   {"mean_fraction_kept": float("%.4g" % (float(d_agree.double().mean().item()) / max(nt - 1, 1)))})


def run_cutovers(plogp, torch, wl, tab, grid, out, nbytes, stream, steps):
    """The cut-over extraction (runs of equal (strategy, s) along m) of the table just tuned."""
    sh = stream.cuda_stream
    n_cells = nbytes // 16
    rows = plogp.plogp_cutover_rows(tab.count, grid)
    d_off = torch.empty(rows + 1, dtype=torch.int64, device="cuda")
    cap = n_cells                      # one record per cell always suffices
    d_runs = torch.empty(cap * 16, dtype=torch.uint8, device="cuda")
    args = (grid, tab.count, out.data_ptr(), plogp.KEY_STRATEGY_AND_SEGMENT, d_off.data_ptr(),
            d_runs.data_ptr(), cap, sh)
    ms, _ = timed_calls(torch, stream, lambda: plogp.plogp_cutovers(*args), steps, 3)
    n_runs = int(d_off[-1].item())
    assert n_runs <= cap, "bench: run buffer too small (%d runs)" % n_runs
    rounds = [plogp.plogp_cutovers_profile(*args, MIN_PER_BATCH) for _ in range(MIN_BATCHES)]
    st = np.median(np.array(rounds), axis=0).tolist()
    # what the extraction itself has to move: the 8-byte key of every cell once, a 16-byte
    # record per run, an 8-byte offset per row
    alg_bytes = 8 * n_cells + 16 * n_runs + 8 * (rows + 1)
    # what it cannot avoid moving: the table keeps key and time in one 16-byte record and HBM
    # moves 64-byte lines, so the whole table is read
    moved = 16 * n_cells + 16 * n_runs + 8 * (rows + 1)
    k_ms = sum(st)
    return hbm_leg(ms, k_ms, alg_bytes, {"runs": n_runs, "stage_ms": {"mark": st[0], "scan": st[1], "emit": st[2]},
                                         "frac_of_peak_whole_records": float("%.3g" % (moved / (k_ms * 1e-3) / HBM_PEAK))})


def run_patterns(cfg, steps):
    """The workload with the rows beyond Tables 1 and 2 switched on as well (Gather ids 13..15,
    Barrier 16, 17: two more planes); their kernel is priced against the HBM write roofline."""
    import torch
    from paper_cs_0408034_amd import plogp
    from plogp_workloads import make_workload
    wl = make_workload(cfg)
    wl.strategy_mask = 0x3FFFF
    work, c = algorithmic_work(wl)
    tab = plogp.plogp_load_tables(wl.sizes, wl.gaps, wl.L)
    grid = plogp.plogp_grid_create(wl.m, wl.P, wl.s, wl.s_cap, wl.dtype_size, wl.strategy_mask)
    nbytes = plogp.plogp_decision_table_bytes(tab.count, grid)
    out = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()
    sh = stream.cuda_stream
    ms, _ = timed_calls(torch, stream, lambda: plogp.plogp_tune_grid(tab, grid, out.data_ptr(), nbytes, sh), steps, 3)
    rounds = [plogp.plogp_tune_grid_profile(tab, grid, out.data_ptr(), nbytes, sh, MIN_PER_BATCH)
              for _ in range(MIN_BATCHES)]
    st = np.median(np.array(rounds), axis=0)
    del out
    grid.free()
    tab.free()
    if st[4] > 0.0005:
        return hbm_leg(ms, float(st[4]), work["more_planes"]["bytes"], {"planes": 4, "kernel": "k_more_planes"})
    # batches whose tables share their sizes: the sweep kernel writes all four planes
    return hbm_leg(ms, float(st[3]), work["sweep"]["bytes"] + work["more_planes"]["bytes"],
                   {"planes": 4, "kernel": "sweep (all four planes)"})


def cpu_sample(cfg, wl):
    """A bounded cut of the same workload for the oracle (a second or two on all cores)."""
    from plogp_workloads import make_workload
    if cfg == 3:
        return make_workload(3, m_slice=slice(0, 1024, 8)), "every 8th m row of config 3 (128 of 1024), all P, all s"
    if cfg == 4:
        return make_workload(4, n_tables=400), "first 400 of the 10 000 tables of config 4, full grid"
    if cfg == 5:
        return make_workload(5, m_slice=slice(0, 4096, 8)), "every 8th m row of config 5 (512 of 4096), all P, all s"
    return wl, "the full %s workload" % wl.name


def run_cpu(cfg, wl):
    """The oracle as it stands, OpenMP over (table, m) rows on the host's cores."""
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
    return {"value": float("%.4g" % (runs * c["nominal_evals"] / dt)), "unit": "evaluations/s", "cores": int(used),
            "kind": "oracle", "sample": "%s, %d run(s), %.1f s wall" % (what, runs, dt),
            "effective_evals_per_s": float("%.4g" % (runs * c["effective_evals"] / dt)),
            "cells_per_s": float("%.4g" % (runs * c["cells"] / dt))}


def bench_config(cfg, steps, warmup, with_cpu, with_next, ceilings=None, mask=None):
    from plogp_workloads import make_workload
    wl = make_workload(cfg)
    if mask is not None:
        wl.strategy_mask = mask
    work, c = algorithmic_work(wl)
    g = run_gpu(wl, steps, warmup, with_next, ceilings_wanted=ceilings is None)
    ceilings = ceilings or g["ceilings"]
    ms, stage_ms = g["ms"], g["stage_ms"]
    fields = ("flops", "flops_executed", "bytes")
    tiny = 0.0005          # ms: two events with nothing between them
    if stage_ms["chain_blocks"] < tiny < stage_ms["sweep"]:
        # one kernel formed the Scatter sums and swept (and, when nothing ran before it, the terms)
        folded = ["chain_blocks", "chain_prefix", "sweep"] + (["terms"] if stage_ms["terms"] < tiny else [])
        work = dict(work)
        work["sweep"] = {f: sum(work[k][f] for k in folded) for f in fields}
        for k in folded[:2] + folded[3:]:
            work[k] = dict.fromkeys(fields, 0)
    elif stage_ms["terms"] < tiny < stage_ms["chain_blocks"]:
        # the terms and the chain sums run in one launch, timed under "chain_blocks"
        work = dict(work)
        work["chain_blocks"] = {f: work["chain_blocks"][f] + work["terms"][f] for f in fields}
        work["terms"] = dict.fromkeys(fields, 0)
    if stage_ms["more_planes"] < tiny < stage_ms["sweep"] and work["more_planes"]["bytes"]:
        # the sweep kernel wrote the Gather and Barrier planes itself
        work = dict(work)
        work["sweep"] = {f: work["sweep"][f] + work["more_planes"][f] for f in fields}
        work["more_planes"] = dict.fromkeys(fields, 0)
    dominant = max(STAGES, key=lambda k: stage_ms[k])
    off = OFFLINE_COUNTERS.get(cfg) if mask is None else None
    stage_of_offline = {"k_row": "sweep", "k_sweep_s": "sweep", "k_batch_t": "sweep", "k_chain_blocks": "chain_blocks"}
    def offline_for(stage):
        if off and stage_of_offline.get(off["kernel"]) == stage:
            return dict(off, cfg=cfg)
        return None
    r4 = lambda v: float("%.4g" % v)
    res = {
        "workload": describe(wl),
        "ms_per_step": ms,
        "value": c["nominal_evals"] / (ms * 1e-3),
        "effective_evals_per_s": r4(c["effective_evals"] / (ms * 1e-3)),
        "cells_per_s": r4(c["cells"] / (ms * 1e-3)),
        "steps_per_batch": g["per_batch"],
        "stage_ms": {k: r4(v) for k, v in stage_ms.items() if v > 0.0005},
        "roofline": roofline_of(dominant, work, stage_ms[dominant], ceilings, offline_for(dominant)),
        "stage_rooflines": {k: roofline_of(k, work, stage_ms[k], ceilings, offline_for(k))
                            for k in STAGES if stage_ms[k] > 0.0005},
        "ceilings": ceilings,
    }
    for k in ("cutovers", "scoring", "robustness"):
        if k in g:
            res[k] = g[k]
    if with_cpu:
        res["cpu_baseline"] = run_cpu(cfg, wl)
    return res


def short(res):
    """What the line keeps of a workload that is not the headline."""
    r = res["roofline"]
    keep = ("kernel", "bound", "achieved", "unit", "frac", "frac_delivered", "frac_executed",
            "frac_of_measured_ceiling", "valu_issue_util", "traffic", "avg_ms")
    out = {"workload": res["workload"], "ms_per_call": float("%.4g" % res["ms_per_step"]),
           "value": float("%.4g" % res["value"]), "cells_per_s": res["cells_per_s"],
           "stage_ms": res["stage_ms"], "roofline": {k: r[k] for k in keep if k in r}}
    others = {k: {f: v[f] for f in ("bound", "frac", "frac_executed") if f in v}
              for k, v in res["stage_rooflines"].items() if k != r["kernel"].split(" ")[0]}
    if others:
        out["other_kernels"] = others
    if "cpu_baseline" in res:
        out["cpu_baseline"] = {k: res["cpu_baseline"][k] for k in ("value", "unit", "cores")}
    return out


def short_next(res):
    out = {}
    for k in ("cutovers", "scoring", "robustness"):
        if k in res:
            v = res[k]
            out[k] = {"ms_per_call": v["ms_per_call"], "kernels_ms": v["kernels_ms"],
                      "hbm_frac": v["roofline"]["frac"]}
            if "frac_of_peak_whole_records" in v:
                out[k]["hbm_frac_whole_records"] = v["frac_of_peak_whole_records"]
    return out


def main():
    global MIN_BATCHES, MIN_PER_BATCH
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100,
                    help="calls per timed batch (at least %d are timed, in %d batches)" % (MIN_PER_BATCH, MIN_BATCHES))
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=4, help="headline workload (1..5)")
    ap.add_argument("--extra", type=str, default="3,5,2", help="other configs to time, or 'none'")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-next", action="store_true", help="skip the steps after the sweep")
    ap.add_argument("--detail", type=str, default=None, help="also write every figure to this JSON file")
    ap.add_argument("--mask", type=lambda v: int(v, 0), default=None,
                    help="strategy mask override (for profiling parts of the path)")
    ap.add_argument("--counters", action="store_true",
                    help="for a rocprofv3 --pmc run, where every dispatch is serialised: one batch of "
                         "three launches of everything, so the counters see each kernel a few times; "
                         "the timings of such a run mean nothing")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one elementwise kernel that copies 256 MiB (known traffic, "
                         "to scale the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.counters:
        MIN_BATCHES, MIN_PER_BATCH = 1, 3
        args.steps, args.warmup = 3, 1
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
    with_next = not args.no_next
    head = bench_config(args.config, args.steps, args.warmup, not args.no_cpu, with_next, None, args.mask)
    r4 = lambda v: float("%.4g" % v)
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
        "timing": {"stat": "median", "batches": MIN_BATCHES, "steps_per_batch": head["steps_per_batch"]},
        "cells_per_s": head["cells_per_s"],
        "effective_evals_per_s": head["effective_evals_per_s"],
        "stage_ms": head["stage_ms"],
        "roofline": head["roofline"],
        "measured_ceilings": {"fp64_fma_tflops": r4(head["ceilings"]["fma_tflops"]),
                              "fill_gbs": r4(head["ceilings"]["store_gbs"]),
                              "spec": {"fp64_vector_tflops": 78.6, "hbm_gbs": 8000.0}},
    }
    if "cpu_baseline" in head:
        line["cpu_baseline"] = head["cpu_baseline"]
    detail = {"cfg%d" % args.config: head}
    extras = [] if args.extra in ("", "none") else [int(v) for v in args.extra.split(",")]
    nxt = {"cfg%d" % args.config: short_next(head)} if with_next else {}
    if with_next and args.mask is None:
        pat = run_patterns(args.config, args.steps)
        detail["cfg%d" % args.config]["more_patterns"] = pat
        nxt["cfg%d" % args.config]["more_patterns"] = {"ms_per_call": pat["ms_per_call"], "kernels_ms": pat["kernels_ms"],
                                                        "hbm_frac": pat["roofline"]["frac"]}
    if extras:
        line["workloads"] = {}
        for cfg in extras:
            if cfg == args.config:
                continue
            res = bench_config(cfg, args.steps, args.warmup, False, with_next and cfg != 2, head["ceilings"])
            detail["cfg%d" % cfg] = res
            line["workloads"]["cfg%d" % cfg] = short(res)
            if with_next and cfg != 2:
                nxt["cfg%d" % cfg] = short_next(res)
                pat = run_patterns(cfg, args.steps)
                detail["cfg%d" % cfg]["more_patterns"] = pat
                nxt["cfg%d" % cfg]["more_patterns"] = {"ms_per_call": pat["ms_per_call"], "kernels_ms": pat["kernels_ms"],
                                                        "hbm_frac": pat["roofline"]["frac"]}
    if nxt:
        line["next"] = nxt
    if args.detail:
        os.makedirs(os.path.dirname(os.path.abspath(args.detail)), exist_ok=True)
        with open(args.detail, "w") as f:
            json.dump(detail, f, indent=1)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
