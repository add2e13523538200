"""Benchmark of the stage-level partition search on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4|c5|c3|c2|c1|c4dense]
                    [--no-cpu-baseline]

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


def updates(N, D, S):
    """Definitional cell-update count of one search."""
    L = min(S, N, D)
    return sum(((N - s + 1) * (N - s + 2) // 2) * ((D - s + 1) * (D - s + 2) // 2)
               for s in range(1, L + 1))


def level_bytes(N, D, esize):
    """Algorithmic bytes of one DP level: the stage-time table read once (entries of `esize`
    bytes), V[s-1] read, V[s] written."""
    return esize * D * N * (N + 1) // 2 + 2 * esize * (N + 1) * D


def make_workload(name):
    from paper_2103_16063_amd import synth
    if name == "c5":
        probs = synth.named_config(5)
        label = "config5 batched sweep: 2048 searches, N=128, D in {8,16,32,64}, S<=16"
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c4")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one 256 MiB device-to-device copy first: the dispatch of known "
                         "size against which rocprofv3's FETCH_SIZE / WRITE_SIZE are scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (D is a search parameter, not a GPU "
              "count); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2103_16063_amd import binding as B
    from paper_2103_16063_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    probs, label = make_workload(args.workload)
    U = sum(updates(p["time_ns"].shape[0], p["n_devices"], p["max_stages"]) for p in probs)
    sess = B.Session(synth.concat_batch(probs))
    esize = 4
    B.rannc_dp_set_timing(sess.h, True)

    def step():
        sess.solve()
        sess.traceback()

    if args.calibration_copy:
        src = torch.zeros(64 << 20, dtype=torch.int32, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    phase = np.zeros(3)
    launches = 0
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
        # per-phase device times of this step (HIP events on the solve's stream); waiting for
        # them also keeps one step in flight at a time, so wall time is per-step latency
        rc, ms, launches = B.rannc_dp_get_timing(sess.h)
        assert rc == B.OK
        phase += ms
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall / args.steps * 1e3
    res = sess.run()
    phase /= args.steps

    # roofline of the dominant kernel (the DP level kernel): algorithmic bytes of one level of
    # every problem in the launch over the average duration of one level launch
    if len(probs) == 1:
        N, D = probs[0]["time_ns"].shape[0], probs[0]["n_devices"]
        lb = level_bytes(N, D, esize)
        per_launch_ms = phase[1] / max(launches, 1)
        achieved = lb / (per_launch_ms * 1e-3) / 1e9
    else:
        # batched: launches are per (level, device-count class); use whole-phase totals
        tot = 0
        for p in probs:
            N, D = p["time_ns"].shape[0], p["n_devices"]
            L = min(p["max_stages"], N, D)
            tot += (L - 1) * level_bytes(N, D, esize)
        per_launch_ms = phase[1] / max(launches, 1)
        achieved = tot / (phase[1] * 1e-3) / 1e9
    out = {
        "metric": "DP cell-updates/sec (definitional count, whole solve incl. table build and traceback)",
        "value": U / (ms_per_step * 1e-3) / 1e9,
        "unit": "G cell-updates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32" if esize == 4 else "u64", "data": "synthetic",
        "config": {"workload": label, "n_problems": len(probs), "cell_updates": U},
        "result": {"opt": int(res["opt"][0]), "n_stages": int(res["n_stages"][0])},
        "phases_ms": {"prefix_and_tables": float(phase[0]), "dp_levels": float(phase[1]),
                      "select": float(phase[2]), "level_launches": int(launches)},
        "level_updates_per_s_G": U / (phase[1] * 1e-3) / 1e9 if phase[1] > 0 else None,
        "roofline": {"bound": "hbm", "kernel": "level_merge_kernel<u32,64>",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "avg_launch_ms": per_launch_ms},
    }
    sess.close()

    if not args.no_cpu_baseline:
        import oracle
        pr = probs[0] if len(probs) == 1 else None
        threads = min(oracle.max_threads(), 16)
        if pr is not None:
            t0 = time.perf_counter()
            o = oracle.solve(pr, n_threads=threads)
            dt = time.perf_counter() - t0
            Ucpu = updates(pr["time_ns"].shape[0], pr["n_devices"], pr["max_stages"])
            sample = "the whole workload once (tables, all levels, traceback)"
            assert o["opt"] == int(res["opt"][0]) and o["n_stages"] == int(res["n_stages"][0])
        else:
            idx = list(range(0, len(probs), len(probs) // 32))[:32]
            t0 = time.perf_counter()
            for q in idx:
                o = oracle.solve(probs[q], n_threads=threads)
                assert o["opt"] == int(res["opt"][q])
            dt = time.perf_counter() - t0
            Ucpu = sum(updates(probs[q]["time_ns"].shape[0], probs[q]["n_devices"],
                               probs[q]["max_stages"]) for q in idx)
            sample = f"{len(idx)} of the {len(probs)} searches (every {len(probs) // 32}th)"
        out["cpu_baseline"] = {"value": Ucpu / dt / 1e9, "unit": "G cell-updates/s",
                               "cores": threads, "kind": "oracle", "sample": sample,
                               "seconds": dt}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
