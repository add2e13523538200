"""Seeded synthetic block chains for the stage-level partition search.

This module only draws numbers: it holds none of the search's arithmetic (no prefix
sums, no stage cost, no memory rule), so that the CPU oracle and the HIP path can both
be fed from it without sharing any code of the method itself.

The chains stand in for the paper's workloads (enlarged BERT and enlarged ResNet block
chains of Sec. IV, and the fine-grained additive-cost regime of Sec. IV-D), which are
not available: a repeating transformer-layer pattern, ResNet-like growth of compute and
parameters with shrinking activations, and heavy-tailed fine-grained units.

Every problem is a dict with
  time_ns, param_bytes, act_bytes : int64[N]  per block, per microbatch at one replica
  n_devices (D), max_stages (S), n_microbatches (MB) : int
  mem_capacity (M) : int bytes
"""
from __future__ import annotations

import math

import numpy as np

MiB = 1 << 20
GiB = 1 << 30


def _problem(t, p, a, D, S, MB, M, name):
    return {
        "name": name,
        "time_ns": np.ascontiguousarray(t, dtype=np.int64),
        "param_bytes": np.ascontiguousarray(p, dtype=np.int64),
        "act_bytes": np.ascontiguousarray(a, dtype=np.int64),
        "n_devices": int(D),
        "max_stages": int(S),
        "n_microbatches": int(MB),
        "mem_capacity": int(M),
    }


def tiny_chain(seed: int = 0, N: int = 16, D: int = 4, S: int = 4, MB: int = 4,
               M: int = 1 * GiB):
    """Config 1: uniform times, parameters and activations; brute-force checkable."""
    g = np.random.default_rng(seed)
    t = g.integers(100_000, 1_000_000, N, endpoint=True)
    p = g.integers(16 * MiB, 256 * MiB, N, endpoint=True)
    a = g.integers(8 * MiB, 128 * MiB, N, endpoint=True)
    return _problem(t, p, a, D, S, MB, M, f"tiny_N{N}_D{D}_S{S}_seed{seed}")


def bert_like_chain(seed: int = 1, layers: int = 24, D: int = 16, S: int = 8,
                    MB: int = 32, M: int = 32 * GiB):
    """Config 2: four block types per transformer layer (attention 1.0x, FFN 2.0x, two
    norm/residual blocks 0.1x of a base time), +-10 % jitter, parameters proportional
    to compute."""
    N = 4 * layers
    g = np.random.default_rng(seed)
    base = int(g.integers(200_000, 400_000, endpoint=True))
    u = g.integers(0, 200, N, endpoint=True)
    mult = np.tile(np.array([10, 20, 1, 1], dtype=np.int64), layers)
    t = base * mult * (900 + u.astype(np.int64)) // 10000
    p = 4096 * t
    a = g.integers(32 * MiB, 96 * MiB, N, endpoint=True)
    return _problem(t, p, a, D, S, MB, M, f"bert_like_N{N}_D{D}_S{S}_seed{seed}")


def resnet_like_chain(N: int = 256, D: int = 32, S: int = 16, MB: int = 64,
                      M: int = 16 * GiB):
    """Config 3: integer recurrences (no randomness): compute x1.01 per block from 5e4 ns,
    parameters x1.015 from 1 MiB, activations x0.99 from 512 MiB."""
    t = np.empty(N, dtype=np.int64)
    p = np.empty(N, dtype=np.int64)
    a = np.empty(N, dtype=np.int64)
    tv, pv, av = 50_000, 1 * MiB, 512 * MiB
    for k in range(N):
        t[k], p[k], a[k] = tv, pv, av
        tv = tv + tv // 100
        pv = pv + 15 * pv // 1000
        av = av - av // 100
    return _problem(t, p, a, D, S, MB, M, f"resnet_like_N{N}_D{D}_S{S}")


def _lognormal_chain(g, N):
    t = np.floor(g.lognormal(math.log(3e5), 0.5, N)).astype(np.int64)
    p = 4 * np.floor(g.lognormal(math.log(64 * MiB), 0.4, N)).astype(np.int64)
    a = g.integers(16 * MiB, 64 * MiB, N, endpoint=True)
    return t, p, a


def enlarged_transformer_chain(seed: int = 3, N: int = 1024, D: int = 64, S: int = 32,
                               MB: int = 128, M: int = 32 * GiB):
    """Config 4: lognormal compute times and 4x lognormal parameter bytes."""
    g = np.random.default_rng(seed)
    t, p, a = _lognormal_chain(g, N)
    return _problem(t, p, a, D, S, MB, M, f"enlarged_N{N}_D{D}_S{S}_seed{seed}")


def batched_sweep(Q: int = 2048, N: int = 128, S: int = 16, M: int = 16 * GiB,
                  seed0: int = 5000):
    """Config 5: Q independent lognormal chains, each with its own seed, device count
    drawn from {8,16,32,64} and microbatch count from {8,16,32,64}."""
    out = []
    for q in range(Q):
        g = np.random.default_rng(seed0 + q)
        D = int(g.choice([8, 16, 32, 64]))
        MB = int(g.choice([8, 16, 32, 64]))
        t, p, a = _lognormal_chain(g, N)
        out.append(_problem(t, p, a, D, S, MB, M, f"sweep_q{q}_N{N}_D{D}"))
    return out


def random_small(seed: int, N: int, D: int, S: int, *, tight: float = 1.0,
                 zero_time_frac: float = 0.0, zero_act: bool = False,
                 tmax: int = 1000):
    """Small random chain for sweeps.  `tight` scales capacity relative to the mean
    per-device share of total memory: below about 1 most instances are infeasible,
    far above 1 memory never binds.  Small `tmax` makes ties frequent."""
    g = np.random.default_rng(seed)
    t = g.integers(0 if zero_time_frac > 0 else 1, tmax, N, endpoint=True)
    if zero_time_frac > 0:
        t = np.where(g.random(N) < zero_time_frac, 0, t)
    p = g.integers(1, 64, N, endpoint=True) * MiB
    a = np.zeros(N, dtype=np.int64) if zero_act else g.integers(1, 64, N, endpoint=True) * MiB
    M = int(tight * (int(p.sum()) + int(a.sum())) / max(1, min(D, N))) + 1
    MB = int(g.choice([1, 2, 4, 8]))
    return _problem(t, p, a, D, S, MB, M, f"rand_N{N}_D{D}_S{S}_seed{seed}")


def with_cut_bytes(problem, seed: int, bandwidth_bytes_per_us: int, lo: int = 1 << 16,
                   hi: int = 16 << 20, zero_frac: float = 0.0):
    """Copy of a problem with the inputs of the communication term added: cut_bytes[k] = bytes of
    the values that cross the cut after block k+1 for one microbatch (uniform in [lo, hi], a
    fraction of them zero), and the bandwidth in bytes per microsecond."""
    g = np.random.default_rng(seed)
    N = problem["time_ns"].shape[0]
    o = g.integers(lo, hi, N, endpoint=True)
    if zero_frac > 0:
        o = np.where(g.random(N) < zero_frac, 0, o)
    out = dict(problem)
    out["cut_bytes"] = np.ascontiguousarray(o, dtype=np.int64)
    out["bandwidth_bytes_per_us"] = int(bandwidth_bytes_per_us)
    out["name"] = problem["name"] + "_comm"
    return out


def with_backward_times(problem, seed: int, tmax: int = 0, ratio: float = 2.0):
    """Copy of a problem with separate backward block times (the split objective of the search:
    "time_ns" then holds the forward times).  tmax > 0: uniform in [0, tmax], independent of the
    forward times; tmax = 0: about `ratio` times the forward time with +-25 % jitter, the usual
    shape of a backward pass."""
    g = np.random.default_rng(seed)
    t = problem["time_ns"]
    N = t.shape[0]
    if tmax > 0:
        tb = g.integers(0, tmax, N, endpoint=True)
    else:
        tb = (t * ratio * (0.75 + 0.5 * g.random(N))).astype(np.int64)
    out = dict(problem)
    out["time_bwd_ns"] = np.ascontiguousarray(tb, dtype=np.int64)
    out["name"] = problem["name"] + "_split"
    return out


def form_stage_case(seed: int, N: int, n_nodes: int, devices_per_node: int, batch_size: int, *,
                    tight: float = 1.0, tmax: int = 2000, layered: bool = False):
    """Inputs of the outer driver of the search (node counts, stage counts and microbatch counts
    tried around the dynamic program): per-SAMPLE block times and transient bytes, persistent
    bytes, the cluster shape and the batch size.  `tight` scales the capacity relative to an even
    share of all bytes of one whole batch over all devices.  `layered` repeats a four-block
    transformer-layer pattern (attention, projection, two MLP halves) instead of i.i.d. blocks."""
    g = np.random.default_rng(seed)
    if layered:
        base_t = np.array([3, 1, 4, 4]) * max(1, tmax // 8)
        base_a = np.array([6, 2, 8, 2])
        base_p = np.array([3, 1, 4, 4])
        k = np.arange(N) % 4
        t = base_t[k] + g.integers(0, max(1, tmax // 16), N, endpoint=True)
        a = (base_a[k] * 64 + g.integers(0, 32, N, endpoint=True)) * 1024
        p = (base_p[k] * 16 + g.integers(0, 8, N, endpoint=True)) * MiB
    else:
        t = g.integers(1, tmax, N, endpoint=True)
        a = g.integers(1, 64, N, endpoint=True) * 64 * 1024
        p = g.integers(1, 64, N, endpoint=True) * MiB
    M = int(tight * (int(p.sum()) + int(a.sum()) * batch_size) / (devices_per_node * n_nodes)) + 1
    return {
        "name": f"form_stage_N{N}_nodes{n_nodes}x{devices_per_node}_BS{batch_size}_seed{seed}",
        "time_per_sample_ns": np.ascontiguousarray(t, dtype=np.int64),
        "act_bytes_per_sample": np.ascontiguousarray(a, dtype=np.int64),
        "param_bytes": np.ascontiguousarray(p, dtype=np.int64),
        "n_nodes": int(n_nodes), "devices_per_node": int(devices_per_node),
        "batch_size": int(batch_size), "mem_capacity": M,
    }


def concat_batch(problems):
    """Concatenate problems into the structure-of-arrays form of the batched call:
    per-problem scalars, block_offset[Q+1], and the three concatenated block arrays."""
    Q = len(problems)
    off = np.zeros(Q + 1, dtype=np.int64)
    for q, pr in enumerate(problems):
        off[q + 1] = off[q] + pr["time_ns"].shape[0]
    cat = lambda k: (np.concatenate([pr[k] for pr in problems]).astype(np.int64)
                     if Q else np.zeros(0, np.int64))
    extra = {}
    if any("cut_bytes" in pr for pr in problems):
        # problems without a communication term get zero bytes on every cut
        extra["cut_bytes"] = np.concatenate(
            [pr.get("cut_bytes", np.zeros(pr["time_ns"].shape[0], np.int64)) for pr in problems]).astype(np.int64)
        extra["bandwidth_bytes_per_us"] = np.array(
            [pr.get("bandwidth_bytes_per_us", 1) for pr in problems], dtype=np.int64)
    if any("time_bwd_ns" in pr for pr in problems):
        assert all("time_bwd_ns" in pr for pr in problems), "split objective: every problem needs backward times"
        extra["time_bwd_ns"] = np.concatenate([pr["time_bwd_ns"] for pr in problems]).astype(np.int64)
    return {
        **extra,
        "n_problems": Q,
        "n_blocks": np.array([pr["time_ns"].shape[0] for pr in problems], dtype=np.int32),
        "n_devices": np.array([pr["n_devices"] for pr in problems], dtype=np.int32),
        "max_stages": np.array([pr["max_stages"] for pr in problems], dtype=np.int32),
        "n_microbatches": np.array([pr["n_microbatches"] for pr in problems], dtype=np.int32),
        "mem_capacity": np.array([pr["mem_capacity"] for pr in problems], dtype=np.int64),
        "block_offset": off,
        "time_ns": cat("time_ns"),
        "param_bytes": cat("param_bytes"),
        "act_bytes": cat("act_bytes"),
    }


def named_config(k: int):
    """Configs 1..5 of the benchmark list (5 returns a list of problems)."""
    if k == 1:
        return tiny_chain()
    if k == 2:
        return bert_like_chain()
    if k == 3:
        return resnet_like_chain()
    if k == 4:
        return enlarged_transformer_chain()
    if k == 5:
        return batched_sweep()
    raise ValueError(k)
