"""Benchmark of the stage-level partition search on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4|c5|c3|c2|c1|c4dense|c4split|c4densesplit]
                    [--no-cpu-baseline] [--no-dense] [--calibration-copy]
    python bench.py --workload formstage32|formstage128|formstage512[split]   (outer driver, Algorithm 2)

A step is one pass of the whole path over one batch of synthetic input that is already resident
in HBM: prefix sums, stage-time / fit tables, every DP level, the choice of the stage count and
the plan recovery.  Prints ONE JSON line.  `value` counts definitional cell updates (one
evaluation of max(V[s-1][i][d'], h(i,j,d-d')) folded into a cell's minimum: the innermost loop
body of Algorithm 1), a number fixed by the shape alone, divided by the wall time of the step.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

HBM_PEAK_GBS = 8000.0
# plain vector ALU rate of the chip: 256 compute units x 4 SIMDs x 16 lanes x 2.4 GHz
ALU_PEAK_TLANEOPS = 256 * 4 * 16 * 2.4e9 / 1e12
# vector instructions per candidate in the split-objective level kernel's loop body (ISA of
# level_split_fast_kernel<64>: 57 per 8 candidates: 16 max, 8 add, 16 compares, 16 selects, 1 move)
SPLIT_VALU_PER_UPDATE = 57 / 8
ESIZE = 4  # bytes per table entry in the 32-bit mode all benchmark configurations run in

# HBM bytes per level-kernel launch as rocprofv3 --pmc measured them (FETCH_SIZE x 2.000 + WRITE_SIZE x
# 1.000 KiB per dispatch, factors from the 256 MiB copy of the same runs).  These are NOT measured by
# this script: each entry names the committed summary it was copied from, and the JSON line repeats
# that name next to the number, so a reader can see where it comes from and whether it is stale.
# Keys: (workload, 64-bit tables, stage times recomputed in some class).  For config 5 a "launch" is
# one of the 32 launches of the level phase (15 levels of the D = 32 and D = 64 classes, the two
# one-launch kernels of the D = 8 and D = 16 classes, tables included): their bytes summed, over 32.
PMC_TRAFFIC = {
    ("c4", False, False): (29.44e6, "profiles/level_merge_config4.md"),
    ("c4", True, False): (48.32e6, "profiles/level_merge_config4_wide.md"),
    ("c4dense", False, False): (113.63e6, "profiles/level_merge_config4_dense.md"),
    ("c4dense", False, True): (9.22e6, "profiles/level_merge_config4_dense_recompute.md"),
    ("c5", False, True): (48.2e6, "profiles/level_merge_config5_batched.md"),
    ("c5", False, False): (811.8e6, "profiles/level_merge_config5_batched_table.md"),
}
# useful vector instructions of the sorted-merge level kernel per (i, j) stage: DP maxima that form
# the bitonic sequence, then log2(DP) compare-exchange stages of DP/2 (max, min) pairs
def merge_valu_per_stage(DP):
    return DP * (DP.bit_length() - 1 + 1)


def updates(N, D, S):
    """Definitional cell-update count of one search."""
    L = min(S, N, D)
    return sum(((N - s + 1) * (N - s + 2) // 2) * ((D - s + 1) * (D - s + 2) // 2)
               for s in range(1, L + 1))


def level_bytes(N, D, esize=ESIZE):
    """Dense equivalent of one DP level: every stage-time entry (i,j,r) of `esize` bytes once, V[s-1]
    read, V[s] written.  What a level would move if nothing could be skipped; never compared with
    the HBM peak (the kernel skips what the method itself skips)."""
    return esize * D * N * (N + 1) // 2 + 2 * esize * (N + 1) * D


def method_work(sess, q, N, D, S_eff, esize, split):
    """The method's own work per DP level of problem q, from the library's table exports of the
    finished solve (fits-in-memory table and value table), in the terms of Algorithm 1: a stage
    (i, j) is visited at level s only if a plan of s-1 stages covers blocks 1..i (the first
    `continue` of the loop body) and the stage fits memory with at most D-s+1 replicas (the second
    one; s-1 devices are spent on the earlier stages); of its stage-time entries only those with
    r <= D-s+1 can be used.  Returns per level s = 2..S_eff:
      entries  stage-time entries (i, j, r) the level has to read, stage by stage
      unit_entries  the same at the granularity the table is stored, skipped and read in: every
               existing column of a (row i, 64-column chunk) unit that holds at least one such stage
      stages   stages (i, j) it has to merge (min-max search) -- lanes with work
      units    (row i, 64-column chunk) pairs with at least one such stage -- waves with work
      rows     rows i of V[s-1] read, cells of V[s] written
      cands    candidates (i, j, d, d') with a finite predecessor and a fitting stage (what the
               split objective must evaluate one by one)"""
    from paper_2103_16063_amd import binding as B
    INF = np.iinfo(np.int64).max
    V = sess.table(B.TABLE_V, q)                      # [S_eff+1][N+1][D+1]
    fit = sess.table(B.TABLE_FIT, q).reshape(-1, D)   # [(j(j-1)/2 + i)][r-1]
    j_of = np.repeat(np.arange(1, N + 1), np.arange(1, N + 1))
    i_of = np.arange(fit.shape[0]) - j_of * (j_of - 1) // 2
    chunk_of = (j_of - 1) >> 6
    out = []
    for s in range(2, S_eff + 1):
        rl = D - s + 1
        row_ok = V[s - 1, :N, D] != INF               # the kernel's test: V[s-1][i][D] finite
        act = row_ok[i_of] & (i_of >= s - 1) & (fit[:, rl - 1] != 0)
        n_act = int(act.sum())
        units, unit_entries, rows = 0, 0, 0
        if n_act:
            ia, ca = i_of[act].astype(np.int64), chunk_of[act].astype(np.int64)
            uid = np.unique(ia * 1024 + ca)
            ui, uc = uid // 1024, uid % 1024
            units = int(uid.shape[0])
            # columns of the unit that exist: j-1 in [max(i, 64c), min(64c+63, N-1)]
            lanes = np.minimum(64 * uc + 63, N - 1) - np.maximum(ui, 64 * uc) + 1
            unit_entries = int(lanes.sum()) * rl
            rows = int(np.unique(ia).shape[0])
        cands = 0
        if split and n_act:
            # per active stage: pairs (d', d) with V[s-1][i][d'] finite, d' < d <= D, d - d' >= rmin
            rmin = D - fit[act].sum(axis=1).astype(np.int64) + 1          # fit is monotone in r
            dlo = np.argmax(V[s - 1, :N, 1:] != INF, axis=1) + 1           # first finite d' per row
            lo = np.maximum(dlo[i_of[act]], s - 1)
            n = D - rmin - lo + 1                                          # d' = lo .. D - rmin
            n = np.maximum(n, 0)
            cands = int((n * (n + 1) // 2).sum())
        out.append({"s": s, "entries": n_act * rl, "unit_entries": unit_entries, "stages": n_act,
                    "units": units, "rows": rows,
                    "cells": (N - s + 1) * (D - s + 1), "cands": cands})
    return out


def make_workload(name):
    from paper_2103_16063_amd import synth
    if name.endswith("split"):
        # Algorithm 1 as printed: separate forward / backward times, backward about twice the forward
        probs, label = make_workload(name[:-5])
        return [synth.with_backward_times(p, 5) for p in probs], label + ", split fwd/bwd objective"
    if name == "c5":
        probs = synth.named_config(5)
        label = "config5 batched sweep: 2048 searches, N=128, D in {8,16,32,64}, S<=16, M=16GiB"
    elif name == "c4dense":
        pr = synth.named_config(4)
        pr["mem_capacity"] = 1 << 50
        probs = [pr]
        label = "config4 shape with unlimited memory (nothing pruned): N=1024, D=64, S<=32"
    else:
        k = int(name[1:])
        probs = [synth.named_config(k)]
        pr = probs[0]
        label = (f"config{k}: N={pr['time_ns'].shape[0]}, D={pr['n_devices']}, "
                 f"S<={pr['max_stages']}, MB={pr['n_microbatches']}, M={pr['mem_capacity'] >> 30}GiB")
    return probs, label


def run_workload(name, steps, warmup, wide=False, algo="auto"):
    """Times `steps` solve+traceback passes of one workload; returns the measurements.  algo: "auto"
    (the library's choice: stage times recomputed inside the level kernel where that applies),
    "table" (the level kernel reads the stage-time table), "recompute"."""
    import torch
    from paper_2103_16063_amd import binding as B
    from paper_2103_16063_amd import synth

    probs, label = make_workload(name)
    U = sum(updates(p["time_ns"].shape[0], p["n_devices"], p["max_stages"]) for p in probs)
    algo_id = {"auto": B.ALGO_AUTO, "table": B.ALGO_MERGE, "recompute": B.ALGO_RECOMPUTE}[algo]
    sess = B.Session(synth.concat_batch(probs), algo=algo_id,
                     max_total_time_ns=(1 << 60) if wide else B.NARROW_MAX_TOTAL_TIME)
    esize = 8 if wide else ESIZE
    split = name.endswith("split")
    DP_of = lambda D: 1 << max(3, int(D - 1).bit_length())

    def step():
        sess.solve()
        sess.traceback()

    def timed_loop(n, with_events):
        """Wall time of n steps, one in flight at a time; with_events: also the per-phase device
        times (HIP events recorded by the library on the solve's stream), summed."""
        ph, nl = np.zeros(3), 0
        t0 = time.perf_counter()
        for _ in range(n):
            step()
            if with_events:
                rc, ms, nl = B.rannc_dp_get_timing(sess.h)  # waits for the step's last event
                assert rc == B.OK
                ph += ms
            else:
                torch.cuda.synchronize()
        torch.cuda.synchronize()
        return time.perf_counter() - t0, ph, nl

    # A batch with several device-count classes runs them on streams of the handle unless the
    # per-phase events are on (they time phases on one stream): then `value` comes from a loop
    # without events and the phase times from a second, shorter one.
    multi = len({1 << max(3, int(p["n_devices"] - 1).bit_length()) for p in probs}) > 1
    B.rannc_dp_set_timing(sess.h, not multi)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    wall, phase, launches = timed_loop(steps, with_events=not multi)
    n_phase = steps
    if multi:
        B.rannc_dp_set_timing(sess.h, True)
        step()
        n_phase = min(steps, 10)
        _, phase, launches = timed_loop(n_phase, with_events=True)
    # latency of one search as a caller sees it: solve call to plan bytes on the host, median of 20
    lat = []
    for _ in range(20):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        res = sess.run()
        lat.append(time.perf_counter() - t0)
    phase /= n_phase
    launches = max(int(launches), 1)
    per_launch_ms = phase[1] / launches
    # ---- the method's own work in the level phase (not timed): from the exports of this solve ----
    rc, info = B.rannc_dp_solve_info(sess.h)   # which level kernel each device-count class ran
    assert rc == B.OK
    kernel_of = {8 << k: info.level_kernel[k] for k in range(4)}
    recompute_any = any(kernel_of[DP_of(p["n_devices"])] == B.KERNEL_MERGE_RECOMPUTE for p in probs)
    tot = {"entries": 0, "unit_entries": 0, "stages": 0, "units": 0, "rows_bytes": 0, "cells_bytes": 0,
           "cands": 0, "valu": 0, "table_bytes": 0, "table_bytes_strict": 0}
    dense_bytes = 0
    for q, p in enumerate(probs):
        N, D = p["time_ns"].shape[0], p["n_devices"]
        S_eff = min(p["max_stages"], N, D)
        DP = DP_of(D)
        recompute = kernel_of[DP] == B.KERNEL_MERGE_RECOMPUTE
        dense_bytes += (S_eff - 1) * level_bytes(N, D, esize)
        for lv in method_work(sess, q, N, D, S_eff, esize, split):
            tot["entries"] += lv["entries"]
            tot["unit_entries"] += lv["unit_entries"]
            tot["stages"] += lv["stages"]
            tot["units"] += lv["units"]
            tot["rows_bytes"] += lv["rows"] * D * esize
            tot["cells_bytes"] += lv["cells"] * esize
            # stage-time table bytes the level has to read (none where the times are recomputed: then one
            # fits-in-memory byte per stage)
            tot["table_bytes"] += 64 * lv["units"] if recompute else esize * lv["unit_entries"]
            tot["table_bytes_strict"] += lv["stages"] if recompute else esize * lv["entries"]
            tot["cands"] += lv["cands"]
            # sorted merge per stage; when the stage times are recomputed, two more instructions for
            # each of the D-s+1 replica counts the level can use
            tot["valu"] += lv["stages"] * merge_valu_per_stage(DP) + (2 * lv["entries"] if recompute else 0)
    sess.close()
    n_tables = 2 if split else 1                  # the split objective reads a backward table too
    n_vals = 3 if split else 1                    # ... and carries two maxima beside each value
    v_bytes = (tot["rows_bytes"] + tot["cells_bytes"]) * n_vals
    own_bytes = tot["table_bytes"] * n_tables + v_bytes
    strict_bytes = tot["table_bytes_strict"] * n_tables + v_bytes
    recompute = recompute_any
    t_levels = phase[1] * 1e-3
    hbm = own_bytes / t_levels / 1e9
    traffic, traffic_src = PMC_TRAFFIC.get((name, bool(wide), bool(recompute)), (None, None))
    if split:
        useful = tot["cands"] * SPLIT_VALU_PER_UPDATE
        alu = useful / t_levels / 1e12
        kernel = "level_split_fast_kernel + split_finalize_kernel (%d-bit values)" % (8 * esize)
    else:
        alu = tot["valu"] / t_levels / 1e12
        kernel = "level_merge_kernel (%d-bit values, %s)" % (
            8 * esize, "stage times recomputed" if recompute else "stage times read from their table")
    frac_hbm, frac_valu = hbm / HBM_PEAK_GBS, alu / ALU_PEAK_TLANEOPS
    bound = "alu" if frac_valu > frac_hbm else "hbm"
    roof = {"bound": bound, "kernel": kernel,
            "achieved": alu if bound == "alu" else hbm,
            "peak": ALU_PEAK_TLANEOPS if bound == "alu" else HBM_PEAK_GBS,
            "unit": "T lane-op/s" if bound == "alu" else "GB/s",
            "frac": max(frac_hbm, frac_valu),
            "frac_hbm": frac_hbm, "frac_valu": frac_valu,
            "traffic": traffic, "traffic_source": traffic_src,
            "avg_launch_ms": per_launch_ms, "launches_per_step": launches,
            "algorithmic_bytes_per_launch": own_bytes / launches,
            "algorithmic_bytes_stage_granularity_per_launch": strict_bytes / launches,
            "frac_hbm_traffic": (traffic / (per_launch_ms * 1e-3) / 1e9 / HBM_PEAK_GBS) if traffic else None,
            "algorithmic_lane_ops_per_launch": (tot["cands"] * SPLIT_VALU_PER_UPDATE if split else tot["valu"]) / launches,
            "stages_visited_per_step": tot["stages"], "table_units_read_per_step": tot["units"],
            "dense_equivalent_bytes_per_launch": dense_bytes / launches,
            "note": "achieved = the method's own bytes (table units that hold a stage Algorithm 1 visits at "
                    "the level, entries r <= D-s+1; rows of V[s-1] read; V[s] written) or useful lane-ops, "
                    "per level launch, over the measured launch time; stage granularity counts only the "
                    "visited stages' own entries; the dense equivalent counts every (i,j,r) and is not "
                    "compared with a peak; traffic is the rocprofv3 counter figure of the named summary"}
    return {"probs": probs, "label": label, "U": U, "ms_per_step": wall / steps * 1e3, "recompute": recompute,
            "latency_ms": float(np.median(lat)) * 1e3,
            "phase": phase, "launches": launches, "res": res, "roofline": roof}


def run_form_stage(name, steps, warmup, cpu_baseline, wide=False):
    """Outer driver (Algorithm 2) end to end: host arrays in, chosen plan on the host, at the
    paper's cluster shape (4 nodes x 8 devices, batch 256, Sec. IV-A).  A step is one call:
    24 searches in three device-count classes plus the host's loops over their results."""
    import torch
    from paper_2103_16063_amd import binding as B
    from paper_2103_16063_amd import synth

    split = name.endswith("split")
    N = int(name[len("formstage"):-5] if split else name[len("formstage"):])
    nn, dn, BS = 4, 8, 256
    c = synth.form_stage_case(7, N, nn, dn, BS, tight=1.3, tmax=2000, layered=True)
    kw = {}
    if split:
        kw["time_bwd_per_sample_ns"] = synth.with_backward_times(
            {"time_ns": c["time_per_sample_ns"], "name": c["name"]}, 5)["time_bwd_ns"]
    fs = B.FormStageSession(N, nn, dn, BS, split=split,
                            max_total_time_ns=(1 << 60) if wide else B.NARROW_MAX_TOTAL_TIME)
    args = (c["time_per_sample_ns"], c["act_bytes_per_sample"], c["param_bytes"], c["mem_capacity"])
    for _ in range(warmup):
        fs.run(*args, **kw)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        rc, out, se, rp = fs.run(*args, **kw)
        assert rc == B.OK
    ms = (time.perf_counter() - t0) / steps * 1e3
    Q = fs.Q
    fs.close()
    # definitional updates of the searches of one call: n = 1, 2, 4 nodes, every MB = 1, 2, 4, ...
    U, n = 0, 1
    while n <= nn:
        D, mb = dn * n, 1
        while mb <= BS // (nn // n):
            U += updates(N, D, D)
            mb *= 2
        n *= 2
    line = {
        "metric": "DP cell-updates/sec (definitional count, outer driver end to end, host arrays in, plan out)",
        "value": U / (ms * 1e-3) / 1e9, "unit": "G cell-updates/s", "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u64" if wide else "u32", "data": "synthetic",
        "config": {"workload": f"outer driver: {nn} nodes x {dn} devices, batch {BS}, N={N} blocks"
                               + (", split fwd/bwd objective" if split else ""),
                   "n_problems": Q, "cell_updates": U},
        "result": {"feasible": int(out.feasible), "n": int(out.n), "n_stages": int(out.n_stages),
                   "n_microbatches": int(out.n_microbatches), "est_iter_ns": int(out.est_iter_ns)},
        "roofline": None,  # bound by launch and copy latency: a few dozen dependent launches of small kernels
    }
    if cpu_baseline:
        import oracle
        t0 = time.perf_counter()
        o = oracle.form_stage(c["time_per_sample_ns"], c["act_bytes_per_sample"], c["param_bytes"], nn, dn, BS,
                              c["mem_capacity"], time_bwd_per_sample_ns=kw.get("time_bwd_per_sample_ns"))
        dt = time.perf_counter() - t0
        assert (o is not None) == bool(out.feasible)
        assert o is None or (o["n_stages"] == out.n_stages and o["est_iter_ns"] == out.est_iter_ns)
        line["cpu_baseline"] = {"value": U / dt / 1e9, "unit": "G cell-updates/s", "cores": 1, "kind": "oracle",
                                "sample": "the whole call once", "seconds": dt}
    return line


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c4")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true",
                    help="skip the extra roofline_dense measurement (c4 workload only)")
    ap.add_argument("--algo", default="auto", choices=["auto", "table", "recompute"],
                    help="level kernel: the library's choice, stage times read from their table, or recomputed")
    ap.add_argument("--no-wide", action="store_true",
                    help="skip the extra measurement of the same workload on 64-bit tables")
    ap.add_argument("--wide", action="store_true",
                    help="use a 64-bit handle (tables of 8-byte values) for the same inputs")
    ap.add_argument("--one-stream", action="store_true",
                    help="keep the device-count classes of a batch on the caller's stream (sets "
                         "RANNC_DP_STREAMS=0), so that a kernel trace shows each kernel on its own")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one 256 MiB device-to-device copy first: the dispatch of known "
                         "size against which rocprofv3's FETCH_SIZE / WRITE_SIZE are scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (D is a search parameter, not a GPU "
              "count); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    if args.one_stream:
        os.environ["RANNC_DP_STREAMS"] = "0"
    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.calibration_copy:
        src = torch.zeros(64 << 20, dtype=torch.int32, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.workload.startswith("formstage"):
        print(json.dumps(run_form_stage(args.workload, args.steps, args.warmup, not args.no_cpu_baseline, args.wide)),
              flush=True)
        return
    m = run_workload(args.workload, args.steps, args.warmup, args.wide, args.algo)
    probs, res, phase = m["probs"], m["res"], m["phase"]
    out = {
        "metric": "DP cell-updates/sec (definitional count, whole solve incl. table build and traceback)",
        "value": m["U"] / (m["ms_per_step"] * 1e-3) / 1e9,
        "unit": "G cell-updates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": m["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u64" if args.wide else "u32", "data": "synthetic",
        "config": {"workload": m["label"], "n_problems": len(probs), "cell_updates": m["U"]},
        "result": {"opt": int(res["opt"][0]), "n_stages": int(res["n_stages"][0])},
        "phases_ms": {"prefix_and_tables": float(phase[0]), "dp_levels": float(phase[1]),
                      "select": float(phase[2]), "level_launches": int(m["launches"])},
        "level_updates_per_s_G": m["U"] / (phase[1] * 1e-3) / 1e9 if phase[1] > 0 else None,
        "latency_to_host_plan_ms": m["latency_ms"],
        "roofline": m["roofline"],
    }
    out["level_kernel"] = "stage times recomputed" if m["recompute"] else "stage times read from their table"
    if m["recompute"] and args.algo == "auto" and not args.no_dense:
        # the same workload with the level kernel that reads the stage-time table (HBM-bound form)
        tm = run_workload(args.workload, max(5, args.steps // 3), 2, algo="table")
        assert int(tm["res"]["opt"][0]) == int(res["opt"][0])
        out["table_mode"] = {"ms_per_step": tm["ms_per_step"], "dp_levels_ms": float(tm["phase"][1]),
                             "prefix_and_tables_ms": float(tm["phase"][0]), "roofline": tm["roofline"]}
    if args.workload == "c4" and not args.no_dense and not args.wide:
        # the same kernels where nothing can be pruned (every stage fits): the streaming case
        for key, algo in (("roofline_dense", "table"), ("roofline_dense_recompute", "recompute")):
            dm = run_workload("c4dense", max(5, args.steps // 5), 2, algo=algo)
            out[key] = dict(dm["roofline"], workload=dm["label"], ms_per_step=dm["ms_per_step"])
    if not args.no_wide and not args.wide and not args.workload.endswith("split"):
        # the same workload on a handle with 64-bit tables (the path inputs with totals above
        # 2^32 - 2 ns take, e.g. the outer driver at the paper's cluster shape)
        wm = run_workload(args.workload, max(5, args.steps // 5), 2, wide=True)
        assert int(wm["res"]["opt"][0]) == int(res["opt"][0])
        out["wide_u64"] = {"dtype": "u64", "ms_per_step": wm["ms_per_step"],
                           "value": wm["U"] / (wm["ms_per_step"] * 1e-3) / 1e9,
                           "dp_levels_ms": float(wm["phase"][1]),
                           "slowdown_vs_u32": wm["ms_per_step"] / m["ms_per_step"],
                           "roofline": wm["roofline"]}

    if not args.no_cpu_baseline:
        import oracle
        ncpu = os.cpu_count()
        threads = min(oracle.max_threads(), 16)

        def time_oracle(n_threads, idx, max_levels=None):
            t0 = time.perf_counter()
            for q in idx:
                o = oracle.solve(probs[q], n_threads=n_threads, max_levels=max_levels)
                if max_levels is None:
                    assert o["opt"] == int(res["opt"][q]) and o["n_stages"] == int(res["n_stages"][q])
            return time.perf_counter() - t0

        if len(probs) == 1:
            idx, sample = [0], "the whole workload once (tables, all levels, traceback)"
            dt = time_oracle(threads, idx)
        else:
            # a batch: every search of it, one search per host thread (the oracle's C calls release the
            # interpreter lock), each checked against the GPU's optimum and stage count
            from concurrent.futures import ThreadPoolExecutor
            idx = list(range(len(probs)))
            sample = f"all {len(probs)} searches, each whole, one search per host thread"

            def one(q):
                o = oracle.solve(probs[q], n_threads=1)
                assert o["opt"] == int(res["opt"][q]) and o["n_stages"] == int(res["n_stages"][q])

            t0 = time.perf_counter()
            with ThreadPoolExecutor(max_workers=threads) as ex:
                list(ex.map(one, idx))
            dt = time.perf_counter() - t0
        Ucpu = sum(updates(probs[q]["time_ns"].shape[0], probs[q]["n_devices"], probs[q]["max_stages"])
                   for q in idx)
        out["cpu_baseline"] = {"value": Ucpu / dt / 1e9, "unit": "G cell-updates/s",
                               "cores": threads, "kind": "oracle", "sample": sample,
                               "seconds": dt, "host_cpus": ncpu}
        # single thread: bounded to about 20 s by the number of levels (one search) or of searches
        rate = Ucpu / dt / threads            # optimistic per-thread rate, only to size the sample
        if len(probs) == 1:
            pr = probs[0]
            N, D = pr["time_ns"].shape[0], pr["n_devices"]
            L, Lmax = 1, min(pr["max_stages"], N, D)
            while L < Lmax and updates(N, D, L + 1) / rate < 20.0:
                L += 1
            dt1 = time_oracle(1, [0], max_levels=None if L == Lmax else L)
            U1 = updates(N, D, L)
            sample1 = ("the whole workload once" if L == Lmax else
                       f"tables and the first {L} of {Lmax} levels of the workload")
        else:
            idx1 = idx[:max(1, int(len(idx) * 20.0 * rate / max(Ucpu, 1)))]
            dt1 = time_oracle(1, idx1)
            U1 = sum(updates(probs[q]["time_ns"].shape[0], probs[q]["n_devices"], probs[q]["max_stages"])
                     for q in idx1)
            sample1 = f"{len(idx1)} of the {len(probs)} searches, each whole"
        out["cpu_baseline_1thread"] = {"value": U1 / dt1 / 1e9, "unit": "G cell-updates/s", "cores": 1,
                                       "kind": "oracle", "sample": sample1, "seconds": dt1,
                                       "host_cpus": ncpu}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
