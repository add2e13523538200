"""Pins for the oracle's outer driver (Algorithm 2 of Sec. III-C): an independent enumeration
from the definition -- every node count, stage count, microbatch count, every plan of exactly S
stages -- with the same selection rule written out separately.  No GPU needed."""
import numpy as np
import pytest

import oracle
from tests import defcheck

INF = defcheck.INF


def enumerate_form_stage(ts, as_, pp, n_nodes, d_node, BS, M, os_=None, w=0):
    N = len(ts)
    n = 1
    while n <= n_nodes:
        D, R = d_node * n, n_nodes // n
        for S in range(d_node * (n - 1) + 1, d_node * n + 1):
            cands = []
            MB = 1
            while MB <= BS // R:
                b = BS // R // MB
                t = [int(x) * b for x in ts]
                a = [int(x) * b for x in as_]
                comm = None if os_ is None else ([int(x) * b for x in os_], w)
                v = defcheck.brute_force_prefix(t, pp, a, S, N, D, M, comm)  # exactly S stages, D devices
                if v != INF:
                    cands.append(((MB + S - 1) * v, MB, v))
                MB *= 2
            if cands:
                est, MB, v = min(cands)  # smallest estimate, then smallest MB
                return {"n": n, "n_stages": S, "n_microbatches": MB, "stage_time_ns": v,
                        "est_iter_ns": est, "devices": D, "replica_factor": R}
        n *= 2
    return None


CASES = []
for seed in range(30):
    g = np.random.default_rng(31_000 + seed)
    CASES.append((seed, int(g.integers(1, 7)), int(g.choice([1, 2, 4])), int(g.integers(1, 3)),
                  int(g.choice([1, 3, 4, 8, 16])), float(g.choice([0.3, 0.6, 1.0, 2.0, 20.0]))))


@pytest.mark.parametrize("seed,N,n_nodes,d_node,BS,tight", CASES)
def test_form_stage_against_enumeration(seed, N, n_nodes, d_node, BS, tight):
    g = np.random.default_rng(seed)
    ts = g.integers(1, 50, N)
    as_ = g.integers(1, 40, N)
    pp = g.integers(1, 100, N)
    M = int(tight * (int(pp.sum()) + int(as_.sum()) * BS) / (d_node * n_nodes)) + 1
    want = enumerate_form_stage(ts, as_, pp, n_nodes, d_node, BS, M)
    got = oracle.form_stage(ts, as_, pp, n_nodes, d_node, BS, M)
    if want is None:
        assert got is None
        return
    assert got is not None
    for k in want:
        assert got[k] == want[k], (k, got[k], want[k])
    # the reported plan has exactly S stages, fits, and attains the value
    R, MB, S, D = got["replica_factor"], got["n_microbatches"], got["n_stages"], got["devices"]
    b = BS // R // MB
    t = [int(x) * b for x in ts]
    a = [int(x) * b for x in as_]
    defcheck.check_plan(t, pp, a, D, S, M, got["stage_time_ns"], S, got["stage_end"], got["replicas"])


def test_form_stage_outcomes_are_mixed():
    kinds = {"none": 0, "n1": 0, "n>1": 0, "mb>1": 0, "s>1": 0}
    for seed, N, n_nodes, d_node, BS, tight in CASES:
        g = np.random.default_rng(seed)
        ts, as_, pp = g.integers(1, 50, N), g.integers(1, 40, N), g.integers(1, 100, N)
        M = int(tight * (int(pp.sum()) + int(as_.sum()) * BS) / (d_node * n_nodes)) + 1
        r = oracle.form_stage(ts, as_, pp, n_nodes, d_node, BS, M)
        if r is None:
            kinds["none"] += 1
            continue
        kinds["n1" if r["n"] == 1 else "n>1"] += 1
        kinds["mb>1"] += r["n_microbatches"] > 1
        kinds["s>1"] += r["n_stages"] > 1
    assert all(v >= 2 for v in kinds.values()), kinds


def test_single_node_single_block_closed_form():
    # one block, one node of 2 devices, batch 4: S = 1, all MB feasible with huge memory;
    # est = MB * ceil(t * floor(4/MB) / 2): MB=1 -> 2t, MB=2 -> 2t, MB=4 -> 2t  => first (MB = 1)
    r = oracle.form_stage([10], [1], [1], 1, 2, 4, 1 << 40)
    assert (r["n"], r["n_stages"], r["n_microbatches"], r["stage_time_ns"], r["est_iter_ns"]) == (1, 1, 1, 20, 20)
    # memory only allows one sample per microbatch per replica pair: act 5 per sample, M = 1 + 5
    r = oracle.form_stage([10], [5], [1], 1, 2, 4, 6)
    assert (r["n_microbatches"], r["stage_time_ns"]) == (2, 10)  # b = 2, ceil(2*5/2) = 5 fits
    assert oracle.form_stage([10], [5], [7], 1, 2, 4, 6) is None


@pytest.mark.parametrize("seed,N,n_nodes,d_node,BS,tight", CASES[:16])
def test_form_stage_with_comm_against_enumeration(seed, N, n_nodes, d_node, BS, tight):
    """The bytes crossing a cut grow with the samples of a microbatch like the times do."""
    g = np.random.default_rng(seed)
    ts, as_, pp = g.integers(1, 50, N), g.integers(1, 40, N), g.integers(1, 100, N)
    os_ = g.integers(0, 30, N)
    w = int(g.choice([700, 1000, 2500]))
    M = int(tight * (int(pp.sum()) + int(as_.sum()) * BS) / (d_node * n_nodes)) + 1
    want = enumerate_form_stage(ts, as_, pp, n_nodes, d_node, BS, M, os_, w)
    got = oracle.form_stage(ts, as_, pp, n_nodes, d_node, BS, M, cut_bytes_per_sample=os_,
                            bandwidth_bytes_per_us=w)
    if want is None:
        assert got is None
        return
    assert got is not None
    for k in want:
        assert got[k] == want[k], (k, got[k], want[k])
    R, MB, S, D = got["replica_factor"], got["n_microbatches"], got["n_stages"], got["devices"]
    b = BS // R // MB
    defcheck.check_plan([int(x) * b for x in ts], pp, [int(x) * b for x in as_], D, S, M,
                        got["stage_time_ns"], S, got["stage_end"], got["replicas"],
                        ([int(x) * b for x in os_], w))


def enumerate_form_stage_split_two_stage_bound(tf, tb, as_, pp, n_nodes, d_node, BS, M):
    """With at most two devices per node count Algorithm 1 as printed is exact (one or two stages:
    nothing is discarded), so the outer loops can be enumerated over the exact split objective."""
    N = len(tf)
    n = 1
    while n <= n_nodes:
        D, R = d_node * n, n_nodes // n
        assert D <= 2
        for S in range(d_node * (n - 1) + 1, d_node * n + 1):
            cands = []
            MB = 1
            while MB <= BS // R:
                b = BS // R // MB
                v = defcheck.brute_force_prefix_split([int(x) * b for x in tf], [int(x) * b for x in tb], pp,
                                                      [int(x) * b for x in as_], S, N, D, M)
                if v != INF:
                    cands.append(((MB + S - 1) * v, MB, v))
                MB *= 2
            if cands:
                est, MB, v = min(cands)
                return {"n": n, "n_stages": S, "n_microbatches": MB, "stage_time_ns": v, "est_iter_ns": est}
        n *= 2
    return None


@pytest.mark.parametrize("seed", range(16))
def test_form_stage_split_objective_small_clusters(seed):
    g = np.random.default_rng(900 + seed)
    N, n_nodes, d_node = int(g.integers(1, 7)), int(g.choice([1, 2])), 1
    BS, tight = int(g.choice([1, 4, 8])), float(g.choice([0.4, 1.0, 3.0]))
    tf, tb = g.integers(1, 50, N), g.integers(1, 90, N)
    as_, pp = g.integers(1, 40, N), g.integers(1, 100, N)
    M = int(tight * (int(pp.sum()) + int(as_.sum()) * BS) / (d_node * n_nodes)) + 1
    want = enumerate_form_stage_split_two_stage_bound(tf, tb, as_, pp, n_nodes, d_node, BS, M)
    got = oracle.form_stage(tf, as_, pp, n_nodes, d_node, BS, M, time_bwd_per_sample_ns=tb)
    if want is None:
        assert got is None
        return
    for k in want:
        assert got[k] == want[k], (k, got[k], want[k])


def test_form_stage_split_equal_halves_doubles_the_value():
    """Backward = forward: every form_stage_dp value doubles and the same plans win, so the outer
    loops make the same choices."""
    for seed, N, n_nodes, d_node, BS, tight in CASES[:12]:
        g = np.random.default_rng(seed)
        ts, as_, pp = g.integers(1, 50, N), g.integers(1, 40, N), g.integers(1, 100, N)
        M = int(tight * (int(pp.sum()) + int(as_.sum()) * BS) / (d_node * n_nodes)) + 1
        a = oracle.form_stage(ts, as_, pp, n_nodes, d_node, BS, M)
        b = oracle.form_stage(ts, as_, pp, n_nodes, d_node, BS, M, time_bwd_per_sample_ns=ts)
        assert (a is None) == (b is None)
        if a is not None:
            for k in ("n", "n_stages", "n_microbatches", "devices", "replica_factor"):
                assert a[k] == b[k]
            assert b["stage_time_ns"] == 2 * a["stage_time_ns"] and b["est_iter_ns"] == 2 * a["est_iter_ns"]
            assert np.array_equal(a["stage_end"], b["stage_end"]) and np.array_equal(a["replicas"], b["replicas"])
