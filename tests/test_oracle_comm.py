"""Pins for the communication term of the stage time (Sec. III-C: a stage's execution time
includes sending its outputs to the following stage; Sec. III-B: estimated from the sizes of the
values and the bandwidth), independent of the oracle's own code.  No GPU needed."""
import numpy as np
import pytest

import oracle
from paper_2103_16063_amd import synth
from tests import defcheck

INF = defcheck.INF


def _solve(pr, **kw):
    return oracle.solve(pr, keep_tables=True, **kw)


def _args(pr):
    return (pr["time_ns"], pr["param_bytes"], pr["act_bytes"])


def _comm(pr):
    return (pr["cut_bytes"], pr["bandwidth_bytes_per_us"])


def small_case(seed, N, D, S, tight, w):
    pr = synth.random_small(seed, N, D, S, tight=tight, tmax=30,
                            zero_time_frac=0.2 if seed % 3 == 0 else 0.0)
    return synth.with_cut_bytes(pr, 900 + seed, w, lo=0, hi=60, zero_frac=0.2 if seed % 4 == 0 else 0.0)


SMALL = []
for seed in range(40):
    g = np.random.default_rng(20_000 + seed)
    SMALL.append((seed, int(g.integers(1, 8, endpoint=True)), int(g.integers(1, 6, endpoint=True)),
                  int(g.integers(1, 5, endpoint=True)), float(g.choice([1.2, 1.4, 1.6, 1.8, 2.0, 2.5, 50.0])),
                  int(g.choice([700, 1000, 3000, 17]))))


@pytest.mark.parametrize("seed,N,D,S,tight,w", SMALL)
def test_brute_force_small_with_comm(seed, N, D, S, tight, w):
    pr = small_case(seed, N, D, S, tight, w)
    r = _solve(pr)
    t, p, a = _args(pr)
    M, comm = pr["mem_capacity"], _comm(pr)
    opt, s_star, _ = defcheck.brute_force(t, p, a, D, S, M, comm)
    assert r["opt"] == opt
    assert r["n_stages"] == s_star
    defcheck.check_plan(t, p, a, D, S, M, r["opt"], r["n_stages"], r["stage_end"], r["replicas"], comm)
    defcheck.check_cells(t, p, a, D, M, r["V"], r["arg_i"], r["arg_d"], comm)


def test_comm_changes_the_answer_often_enough():
    """The sweep must contain instances whose optimum, stage count or plan differs from the same
    instance without the term, else it pins less than it seems to."""
    differs = plans = 0
    for seed, N, D, S, tight, w in SMALL:
        pr = small_case(seed, N, D, S, tight, w)
        bare = {k: v for k, v in pr.items() if k not in ("cut_bytes", "bandwidth_bytes_per_us")}
        r, r0 = _solve(pr), _solve(bare)
        differs += r["opt"] != r0["opt"]
        plans += (r["opt"] != INF and (not np.array_equal(r["stage_end"], r0["stage_end"])
                                       or not np.array_equal(r["replicas"], r0["replicas"])))
    assert differs >= 8 and plans >= 4, (differs, plans)


def test_worked_example():
    """Two blocks that cannot share a stage (persistent bytes 5 + 5 > M = 5), three devices,
    1000 bytes/us so that one byte costs one ns: the plans are
      replicas (1,2): max(9 + 2, ceil(20/2)) = 11      replicas (2,1): max(ceil(9/2) + 1, 20) = 20
    and the bytes after the LAST block never count."""
    pr = {"name": "worked", "time_ns": np.array([9, 20]), "param_bytes": np.array([5, 5]),
          "act_bytes": np.array([0, 0]), "n_devices": 3, "max_stages": 2, "n_microbatches": 1,
          "mem_capacity": 5, "cut_bytes": np.array([2, 10**9]), "bandwidth_bytes_per_us": 1000}
    r = _solve(pr)
    assert r["opt"] == 11 and r["n_stages"] == 2
    assert r["stage_end"].tolist() == [1, 2] and r["replicas"].tolist() == [1, 2]
    pr["cut_bytes"] = np.array([12, 0])  # now (1,2) costs 21 and (2,1) costs max(5 + 6, 20) = 20
    r = _solve(pr)
    assert r["opt"] == 20 and r["replicas"].tolist() == [2, 1]
    pr["bandwidth_bytes_per_us"] = 7     # 12 bytes at 7 B/us: ceil(12000/7) = 1715, halved 858
    r = _solve(pr)
    assert r["opt"] == 863 and r["replicas"].tolist() == [2, 1]   # ceil(9/2) + ceil(12000/14)


def test_tables_against_definition_with_comm():
    pr = small_case(5, 7, 6, 3, 1.0, 700)
    pr = synth.with_cut_bytes(synth.random_small(5, 9, 6, 3, tight=1.0), 11, 700, lo=0, hi=5000)
    r = _solve(pr)
    t, p, a = _args(pr)
    N, D = 9, 6
    for j in range(1, N + 1):
        for i in range(j):
            for rr in range(1, D + 1):
                e = oracle.table_index(j, i, rr, D)
                assert int(r["cost"][e]) == defcheck.stage_time(t, i, j, rr, _comm(pr))
                assert bool(r["fit"][e]) == (defcheck.stage_mem(p, a, i, j, rr) <= pr["mem_capacity"])


def test_prefix_cells_against_enumeration_with_comm():
    pr = synth.with_cut_bytes(synth.random_small(77, 7, 5, 4, tight=1.1, tmax=50), 3, 1000, lo=0, hi=40)
    r = _solve(pr)
    t, p, a = _args(pr)
    for s in range(1, 5):
        for j in range(1, 8):
            for d in range(1, 6):
                want = defcheck.brute_force_prefix(t, p, a, s, j, d, pr["mem_capacity"], _comm(pr))
                assert int(r["V"][s, j, d]) == want, (s, j, d)


@pytest.mark.parametrize("seed", range(6))
def test_comm_invariants(seed):
    base = synth.random_small(300 + seed, 14, 7, 5, tight=2.0, tmax=400)
    pr = synth.with_cut_bytes(base, seed, 1000, lo=0, hi=300)
    r0, r = _solve(base), _solve(pr)
    # sending costs time: no cell gets better, and cells of one stage over ALL blocks do not change
    assert (r["V"] >= r0["V"]).all()
    assert np.array_equal(r["V"][1, 14, :], r0["V"][1, 14, :])
    # zero bytes on every cut is the same as no term at all, whatever the bandwidth
    z = dict(pr); z["cut_bytes"] = np.zeros(14, np.int64); z["bandwidth_bytes_per_us"] = 3
    rz = _solve(z)
    for k in ("V", "arg_i", "arg_d", "cost", "fit"):
        assert np.array_equal(rz[k], r0[k])
    # more bandwidth never hurts; unbounded bandwidth leaves at most 1 ns per cut
    prev = None
    for w in (1, 10, 1000, 10**6, 10**15):
        q = dict(pr); q["bandwidth_bytes_per_us"] = w
        v = _solve(q)["V"]
        if prev is not None:
            assert (v <= prev).all()
        prev = v
    fin = r0["V"] != INF
    assert (prev[fin] <= r0["V"][fin] + 1).all()
    # V stays non-increasing in the device total (what the merge form of the level relies on)
    V = r["V"]
    for s in range(1, V.shape[0]):
        for j in range(1, 15):
            row = V[s, j, 1:]
            assert all(row[k] >= row[k + 1] for k in range(len(row) - 1))


def test_comm_rejects_bad_input():
    pr = synth.with_cut_bytes(synth.random_small(1, 5, 3, 3), 1, 1000)
    bad = dict(pr); bad["cut_bytes"] = pr["cut_bytes"].copy(); bad["cut_bytes"][2] = -1
    with pytest.raises(oracle.OracleError):
        oracle.solve(bad)
    bad = dict(pr); bad["bandwidth_bytes_per_us"] = 0
    with pytest.raises(oracle.OracleError):
        oracle.solve(bad)
    bad = dict(pr); bad["cut_bytes"] = pr["cut_bytes"].copy(); bad["cut_bytes"][0] = 1 << 61
    with pytest.raises(oracle.OracleError):
        oracle.solve(bad)
    bad = dict(pr); bad["cut_bytes"] = pr["cut_bytes"][:-1]
    with pytest.raises(oracle.OracleError):
        oracle.solve(bad)
