"""ctypes front end of the CPU oracle (test infrastructure, never used by the product path).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this package.
It compiles oracle/rannc_dp_oracle.c with gcc on first use and wraps its entry points with
numpy arrays.  Nothing here is shared with the HIP path.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rannc_dp_oracle.c")
_LIB = os.path.join(_HERE, "librannc_dp_oracle.so")
INF = np.iinfo(np.int64).max

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle shared library (gcc -O2 -fopenmp)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t))


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        i32, i64, u8 = C.c_int32, C.c_int64, C.c_uint8
        pi32, pi64, pu8 = C.POINTER(i32), C.POINTER(i64), C.POINTER(u8)
        L.rannc_oracle_prefix.argtypes = [i32, pi64, pi64]
        L.rannc_oracle_prefix.restype = C.c_int
        L.rannc_oracle_table_entries.argtypes = [i32, i32]
        L.rannc_oracle_table_entries.restype = C.c_size_t
        L.rannc_oracle_tables.argtypes = [i32, i32, pi64, pi64, pi64, i64, pi64, i64, pi64, pu8]
        L.rannc_oracle_tables.restype = C.c_int
        L.rannc_oracle_dp.argtypes = [i32, i32, i32, pi64, pu8, pi64, pi32, pi32, i32]
        L.rannc_oracle_dp.restype = C.c_int
        L.rannc_oracle_dp_split.argtypes = [i32, i32, i32, pi64, pi64, pu8, pi64, pi64, pi64, pi32, pi32, i32]
        L.rannc_oracle_dp_split.restype = C.c_int
        L.rannc_oracle_dp_pruned.argtypes = [i32, i32, i32, pi64, pu8, pi64, pi64]
        L.rannc_oracle_dp_pruned.restype = C.c_int
        L.rannc_oracle_compact.argtypes = [i32, pi64, pi64, pi64, i32, i64, i32, pi32, pi32]
        L.rannc_oracle_compact.restype = C.c_int
        L.rannc_oracle_select.argtypes = [i32, i32, i32, pi64, pi64, pi32]
        L.rannc_oracle_select.restype = C.c_int
        L.rannc_oracle_traceback.argtypes = [i32, i32, i32, pi32, pi32, i32, pi32, pi32]
        L.rannc_oracle_traceback.restype = C.c_int
        L.rannc_oracle_est_iter_ns.argtypes = [i64, i32, i32]
        L.rannc_oracle_est_iter_ns.restype = i64
        L.rannc_oracle_max_threads.argtypes = []
        L.rannc_oracle_max_threads.restype = C.c_int
        _lib = L
    return _lib


class OracleError(RuntimeError):
    pass


def _chk(rc, what):
    if rc != 0:
        raise OracleError(f"{what}: oracle error {rc}")


def max_threads() -> int:
    return int(lib().rannc_oracle_max_threads())


def prefix(x) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.int64)
    X = np.empty(x.shape[0] + 1, dtype=np.int64)
    _chk(lib().rannc_oracle_prefix(x.shape[0], _p(x, C.c_int64), _p(X, C.c_int64)), "prefix")
    return X


def tables(T, P, A, D: int, M: int, cut_bytes=None, bandwidth_bytes_per_us: int = 0):
    """cost (int64) and fit (uint8), packed as ((j*(j-1)/2 + i)*D + (r-1)).  cut_bytes[k-1] =
    bytes crossing the cut after block k (None: no communication term)."""
    N = T.shape[0] - 1
    n = lib().rannc_oracle_table_entries(N, D)
    cost = np.empty(n, dtype=np.int64)
    fit = np.empty(n, dtype=np.uint8)
    o = None
    if cut_bytes is not None:
        o = np.ascontiguousarray(cut_bytes, dtype=np.int64)
        if o.shape[0] != N:
            raise OracleError("cut_bytes must have one entry per block")
    _chk(lib().rannc_oracle_tables(N, D, _p(T, C.c_int64), _p(P, C.c_int64), _p(A, C.c_int64),
                                   int(M), _p(o, C.c_int64) if o is not None else None,
                                   int(bandwidth_bytes_per_us), _p(cost, C.c_int64),
                                   _p(fit, C.c_uint8)), "tables")
    return cost, fit


def table_index(j, i, r, D):
    return (j * (j - 1) // 2 + i) * D + (r - 1)


def dp(N: int, D: int, n_levels: int, cost, fit, n_threads: int = 1):
    shape = (n_levels + 1, N + 1, D + 1)
    V = np.empty(shape, dtype=np.int64)
    ai = np.empty(shape, dtype=np.int32)
    ad = np.empty(shape, dtype=np.int32)
    _chk(lib().rannc_oracle_dp(N, D, n_levels, _p(cost, C.c_int64), _p(fit, C.c_uint8),
                               _p(V, C.c_int64), _p(ai, C.c_int32), _p(ad, C.c_int32),
                               int(n_threads)), "dp")
    return V, ai, ad


def dp_split(N: int, D: int, n_levels: int, costf, costb, fit, n_threads: int = 1):
    """Algorithm 1 with separate forward / backward maxima: V, TF, TB, arg_i, arg_d."""
    shape = (n_levels + 1, N + 1, D + 1)
    V, TF, TB = (np.empty(shape, dtype=np.int64) for _ in range(3))
    ai = np.empty(shape, dtype=np.int32)
    ad = np.empty(shape, dtype=np.int32)
    _chk(lib().rannc_oracle_dp_split(N, D, n_levels, _p(costf, C.c_int64), _p(costb, C.c_int64),
                                     _p(fit, C.c_uint8), _p(V, C.c_int64), _p(TF, C.c_int64),
                                     _p(TB, C.c_int64), _p(ai, C.c_int32), _p(ad, C.c_int32),
                                     int(n_threads)), "dp_split")
    return V, TF, TB, ai, ad


def dp_pruned(N: int, D: int, S: int, cost, fit):
    """Algorithm 1 for exactly S stages with its printed pruning (trimmed loop ranges, d_min):
    returns (V, cells visited, candidates scanned, final d_min).  A study; see the C source."""
    V = np.empty((S + 1, N + 1, D + 1), dtype=np.int64)
    stats = np.zeros(3, dtype=np.int64)
    _chk(lib().rannc_oracle_dp_pruned(N, D, S, _p(cost, C.c_int64), _p(fit, C.c_uint8),
                                      _p(V, C.c_int64), _p(stats, C.c_int64)), "dp_pruned")
    return V, int(stats[0]), int(stats[1]), int(stats[2])


def select(V):
    n_levels, N, D = V.shape[0] - 1, V.shape[1] - 1, V.shape[2] - 1
    opt = C.c_int64()
    ns = C.c_int32()
    _chk(lib().rannc_oracle_select(N, D, n_levels, _p(V, C.c_int64), C.byref(opt), C.byref(ns)),
         "select")
    return int(opt.value), int(ns.value)


def traceback(ai, ad, n_stages: int, max_slots: int):
    N, D = ai.shape[1] - 1, ai.shape[2] - 1
    se = np.empty(max_slots, dtype=np.int32)
    rp = np.empty(max_slots, dtype=np.int32)
    _chk(lib().rannc_oracle_traceback(N, D, n_stages, _p(ai, C.c_int32), _p(ad, C.c_int32),
                                      max_slots, _p(se, C.c_int32), _p(rp, C.c_int32)),
         "traceback")
    return se, rp


def compact(time_ns, param_bytes, act_bytes, k: int, mem_capacity: int, max_passes: int = 0):
    """Compaction step of the block-level phase on a chain (Sec. III-B): returns the ends of the
    resulting groups (1-based counts of input groups, the last one = G) and their summed time,
    persistent and transient bytes -- the block arrays the stage-level search takes.
    max_passes = 0: the walk over the groups listed by time is repeated (on the groups as they
    then stand) until k groups are left or a walk merges nothing; n > 0: at most n walks."""
    t = np.ascontiguousarray(time_ns, dtype=np.int64)
    p = np.ascontiguousarray(param_bytes, dtype=np.int64)
    a = np.ascontiguousarray(act_bytes, dtype=np.int64)
    G = int(t.shape[0])
    end = np.empty(G, dtype=np.int32)
    n = C.c_int32()
    _chk(lib().rannc_oracle_compact(G, _p(t, C.c_int64), _p(p, C.c_int64), _p(a, C.c_int64), int(k),
                                    int(mem_capacity), int(max_passes), C.byref(n), _p(end, C.c_int32)),
         "compact")
    end = end[:n.value].copy()
    lo = np.concatenate(([0], end[:-1]))
    T, P, A = prefix(t), prefix(p), prefix(a)
    return end, T[end] - T[lo], P[end] - P[lo], A[end] - A[lo]


def est_iter_ns(opt: int, n_stages: int, MB: int) -> int:
    return int(lib().rannc_oracle_est_iter_ns(int(opt), int(n_stages), int(MB)))


def solve(problem, n_threads: int = 1, keep_tables: bool = False, max_levels=None):
    """Whole path for one problem dict (see the input generator module for its keys).

    Returns a dict with opt, n_stages, est_iter_ns, stage_end[S], replicas[S] and, with
    keep_tables, T/P/A, cost, fit, V, arg_i, arg_d.  max_levels bounds the number of levels
    computed (used only to time a bounded sample of a large search).  A problem that carries
    "time_bwd_ns" is searched with the split objective of Algorithm 1 ("time_ns" is then the
    forward time; the communication term, if any, belongs to the forward pass): opt is the
    sum of the largest forward and the largest backward stage time, also returned as max_fwd,
    max_bwd, and keep_tables adds cost_bwd, TF, TB."""
    t, p, a = problem["time_ns"], problem["param_bytes"], problem["act_bytes"]
    N = int(t.shape[0])
    D, S = int(problem["n_devices"]), int(problem["max_stages"])
    MB, M = int(problem["n_microbatches"]), int(problem["mem_capacity"])
    if D < 1 or S < 1 or MB < 1 or M < 0:
        raise OracleError("bad scalar argument")
    T, P, A = prefix(t), prefix(p), prefix(a)
    cost, fit = tables(T, P, A, D, M, problem.get("cut_bytes"),
                       int(problem.get("bandwidth_bytes_per_us", 0)))
    n_levels = min(S, N, D)
    if max_levels is not None:
        n_levels = min(n_levels, int(max_levels))
    split = "time_bwd_ns" in problem
    if split:
        costb, _ = tables(prefix(problem["time_bwd_ns"]), P, A, D, M)
        V, TF, TB, ai, ad = dp_split(N, D, n_levels, cost, costb, fit, n_threads)
    else:
        V, ai, ad = dp(N, D, n_levels, cost, fit, n_threads)
    opt, ns = select(V)
    se, rp = traceback(ai, ad, ns, S)
    out = {"opt": opt, "n_stages": ns, "est_iter_ns": est_iter_ns(opt, ns, MB),
           "stage_end": se, "replicas": rp, "n_levels": n_levels}
    if split:
        out.update(max_fwd=int(TF[ns, N, D]) if ns else INF, max_bwd=int(TB[ns, N, D]) if ns else INF)
    if keep_tables:
        out.update(T=T, P=P, A=A, cost=cost, fit=fit, V=V, arg_i=ai, arg_d=ad)
        if split:
            out.update(cost_bwd=costb, TF=TF, TB=TB)
    return out


def form_stage(time_per_sample_ns, act_bytes_per_sample, param_bytes, n_nodes: int,
               devices_per_node: int, batch_size: int, mem_capacity: int, n_threads: int = 1,
               cut_bytes_per_sample=None, bandwidth_bytes_per_us: int = 0,
               time_bwd_per_sample_ns=None):
    """Outer driver of the search (Algorithm 2 "form_stage" of Sec. III-C), loops in the paper's
    order: node count n = 1, 2, 4, ... <= n_nodes; D = devices_per_node * n devices, replica factor
    R = n_nodes / n; stage count S ascending over (devices_per_node*(n-1), devices_per_node*n]; for
    each S every microbatch count MB = 1, 2, 4, ... <= floor(batch_size / R) is tried with
    form_stage_dp for EXACTLY S stages (Algorithm 1's answer V[S][|B|][D]); the first S with a
    feasible MB returns the best of its solutions.

    Readings (the paper leaves them open): a block's time and transient bytes grow linearly with
    the samples of a microbatch on one pipeline replica, b = floor(batch_size / R / MB), its
    persistent bytes do not (the bytes crossing a cut, if given, grow the same way); with
    time_bwd_per_sample_ns every form_stage_dp call is Algorithm 1 as printed (forward and
    backward maxima carried separately, time_per_sample_ns being the forward time) and V is the
    sum of the two maxima; "best" = smallest (MB + S - 1) * V, the time of one synchronous
    pipeline iteration (Fig. 1), the first found among equals (smallest MB); R is the integer
    quotient.  The DP for one (n, MB) yields every exact-S value at once, so it is memoised.

    Returns None if infeasible, else a dict with n, devices (D), replica_factor (R), n_stages (S),
    n_microbatches (MB), stage_time_ns (V), est_iter_ns, stage_end[S], replicas[S] (d_i, before
    the factor R)."""
    ts = np.ascontiguousarray(time_per_sample_ns, dtype=np.int64)
    as_ = np.ascontiguousarray(act_bytes_per_sample, dtype=np.int64)
    pp = np.ascontiguousarray(param_bytes, dtype=np.int64)
    os_ = (None if cut_bytes_per_sample is None
           else np.ascontiguousarray(cut_bytes_per_sample, dtype=np.int64))
    tbs = (None if time_bwd_per_sample_ns is None
           else np.ascontiguousarray(time_bwd_per_sample_ns, dtype=np.int64))
    N = int(ts.shape[0])
    if n_nodes < 1 or devices_per_node < 1 or batch_size < 1 or mem_capacity < 0:
        raise OracleError("bad scalar argument")
    memo = {}

    def dp_tables(n, MB):
        if (n, MB) not in memo:
            D = devices_per_node * n
            R = n_nodes // n
            b = batch_size // R // MB
            T, P, A = prefix(ts * b), prefix(pp), prefix(as_ * b)
            cost, fit = tables(T, P, A, D, mem_capacity, None if os_ is None else os_ * b,
                               bandwidth_bytes_per_us)
            if tbs is None:
                memo[(n, MB)] = dp(N, D, min(D, N), cost, fit, n_threads)
            else:
                costb, _ = tables(prefix(tbs * b), P, A, D, mem_capacity)
                V, _, _, ai, ad = dp_split(N, D, min(D, N), cost, costb, fit, n_threads)
                memo[(n, MB)] = (V, ai, ad)
        return memo[(n, MB)]

    n = 1
    while n <= n_nodes:
        D = devices_per_node * n
        R = n_nodes // n
        for S in range(devices_per_node * (n - 1) + 1, devices_per_node * n + 1):
            best = None
            MB = 1
            while MB <= batch_size // R:
                if S <= min(N, D):
                    V, ai, ad = dp_tables(n, MB)
                    v = int(V[S, N, D])
                    if v != INF:
                        est = (MB + S - 1) * v
                        if best is None or est < best["est_iter_ns"]:
                            se, rp = traceback(ai, ad, S, S)
                            best = {"n": n, "devices": D, "replica_factor": R, "n_stages": S,
                                    "n_microbatches": MB, "stage_time_ns": v, "est_iter_ns": est,
                                    "stage_end": se, "replicas": rp}
                MB *= 2
            if best is not None:
                return best
        n *= 2
    return None
