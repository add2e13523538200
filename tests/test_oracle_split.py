"""Pins for the oracle's run of Algorithm 1 as printed (Sec. III-C): forward and backward maxima
carried separately, candidates valued by their sum.  From the third level on that is a heuristic,
so the pins are what the mathematics still fixes: levels 1 and 2 are exact; equal or all-zero
backward times reduce to the (pinned) min-max search; every value is the value of the plan stored
with it and never below the exact minimum; and a worked example in which the heuristic misses the
optimum by the margin that follows from its steps.  No GPU needed."""
import numpy as np
import pytest

import oracle
from paper_2103_16063_amd import synth
from tests import defcheck

INF = defcheck.INF


def split_case(seed, N, D, S, tight, tmax=30, comm=False):
    pr = synth.with_backward_times(synth.random_small(seed, N, D, S, tight=tight, tmax=tmax), 400 + seed, tmax)
    if comm:
        pr = synth.with_cut_bytes(pr, 70 + seed, 1000, lo=0, hi=tmax)
    return pr


def _comm(pr):
    return (pr["cut_bytes"], pr["bandwidth_bytes_per_us"]) if "cut_bytes" in pr else None


def _solve(pr):
    return oracle.solve(pr, keep_tables=True)


SMALL = []
for seed in range(36):
    g = np.random.default_rng(40_000 + seed)
    SMALL.append((seed, int(g.integers(1, 8, endpoint=True)), int(g.integers(1, 6, endpoint=True)),
                  int(g.integers(1, 5, endpoint=True)), float(g.choice([1.2, 1.5, 2.0, 3.0, 50.0])), seed % 3 == 0))


@pytest.mark.parametrize("seed,N,D,S,tight,comm", SMALL)
def test_values_are_plan_values_bounded_by_the_exact_minimum(seed, N, D, S, tight, comm):
    pr = split_case(seed, N, D, S, tight, comm=comm)
    r = _solve(pr)
    tf, tb, p, a, M = pr["time_ns"], pr["time_bwd_ns"], pr["param_bytes"], pr["act_bytes"], pr["mem_capacity"]
    V, TF, TB = r["V"], r["TF"], r["TB"]
    for s in range(1, V.shape[0]):
        for j in range(0, N + 1):
            for d in range(0, D + 1):
                v = int(V[s, j, d])
                exact = (defcheck.brute_force_prefix_split(tf, tb, p, a, s, j, d, M, _comm(pr))
                         if j >= 1 and d >= 1 else INF)
                assert (v == INF) == (exact == INF), (s, j, d)   # feasibility is exact at every level
                if v == INF:
                    assert int(TF[s, j, d]) == INF and int(TB[s, j, d]) == INF
                    assert int(r["arg_i"][s, j, d]) == -1 and int(r["arg_d"][s, j, d]) == -1
                    continue
                assert v >= exact, (s, j, d)
                if s <= 2:
                    assert v == exact, (s, j, d)                 # one or two stages: nothing is discarded
                bounds, reps = defcheck.walk_back(r["arg_i"], r["arg_d"], s, j, d)
                ok, mf, mb = defcheck.plan_value_split(tf, tb, p, a, M, bounds, reps, _comm(pr))
                # a prefix plan sends after its last stage too unless it ends the chain: plan_value_split
                # applies the term by the stage's end, which is what the table holds
                assert ok and (mf, mb) == (int(TF[s, j, d]), int(TB[s, j, d])) and mf + mb == v, (s, j, d)
    # the reported answer
    col = [int(V[s, N, D]) for s in range(1, V.shape[0])]
    want = min(col) if col else INF
    assert r["opt"] == want
    if want == INF:
        assert r["n_stages"] == 0
    else:
        assert r["n_stages"] == 1 + col.index(want)
        assert r["max_fwd"] + r["max_bwd"] == r["opt"]
        ns = r["n_stages"]
        bounds, reps = defcheck.walk_back(r["arg_i"], r["arg_d"], ns, N, D)
        assert bounds[1:] == r["stage_end"][:ns].tolist() and reps == r["replicas"][:ns].tolist()
        assert sum(reps) == D and bounds[-1] == N


@pytest.mark.parametrize("seed,N,D,S,tight,comm", SMALL)
def test_second_run_of_the_steps(seed, N, D, S, tight, comm):
    pr = split_case(seed, N, D, S, tight, comm=comm)
    r = _solve(pr)
    cells = defcheck.split_steps(pr["time_ns"], pr["time_bwd_ns"], pr["param_bytes"], pr["act_bytes"], D,
                                 pr["mem_capacity"], r["V"].shape[0] - 1, _comm(pr))
    for s in range(r["V"].shape[0]):
        for j in range(N + 1):
            for d in range(D + 1):
                got = tuple(int(r[k][s, j, d]) for k in ("V", "TF", "TB", "arg_i", "arg_d"))
                want = cells.get((s, j, d), (INF, INF, INF, -1, -1))
                assert got == want, (s, j, d)


def test_sweep_is_not_trivial():
    """The sweep must hold cells where the heuristic is above the exact minimum, and feasible as
    well as infeasible instances."""
    above = feas = infeas = multi = 0
    for seed, N, D, S, tight, comm in SMALL:
        pr = split_case(seed, N, D, S, tight, comm=comm)
        r = _solve(pr)
        feas += r["opt"] != INF
        infeas += r["opt"] == INF
        multi += r["n_stages"] > 1
        V = r["V"]
        for s in range(3, V.shape[0]):
            for j in range(1, N + 1):
                for d in range(1, D + 1):
                    if int(V[s, j, d]) != INF:
                        above += int(V[s, j, d]) > defcheck.brute_force_prefix_split(
                            pr["time_ns"], pr["time_bwd_ns"], pr["param_bytes"], pr["act_bytes"], s, j, d,
                            pr["mem_capacity"], _comm(pr))
    assert feas >= 10 and infeas >= 3 and multi >= 5 and above >= 1, (feas, infeas, multi, above)


def test_worked_example_where_one_pair_per_cell_loses():
    """Four blocks, three devices, three stages of one replica each, memory not binding.
    forward 3 1 2 4, backward 1 3 2 4.  Two stages over blocks 1..3: {1}{2,3} gives (max fwd, max bwd)
    = (3, 5), {1,2}{3} gives (4, 4): both sum to 8, the first scanned (split after block 1) stays.
    Adding block 4 (4, 4) as the third stage then gives (4, 5) = 9, although {1,2}{3}{4} is worth
    (4, 4) = 8; the other candidate {1}{2}{3,4} is worth (6, 6) = 12."""
    N = 4
    pr = {"name": "worked_split", "time_ns": np.array([3, 1, 2, 4]), "time_bwd_ns": np.array([1, 3, 2, 4]),
          "param_bytes": np.zeros(N, np.int64), "act_bytes": np.zeros(N, np.int64), "n_devices": 3,
          "max_stages": 3, "n_microbatches": 1, "mem_capacity": 0}
    r = _solve(pr)
    assert (int(r["V"][2, 3, 2]), int(r["TF"][2, 3, 2]), int(r["TB"][2, 3, 2])) == (8, 3, 5)
    assert (int(r["arg_i"][2, 3, 2]), int(r["arg_d"][2, 3, 2])) == (1, 1)
    assert (int(r["V"][3, 4, 3]), int(r["TF"][3, 4, 3]), int(r["TB"][3, 4, 3])) == (9, 4, 5)
    assert defcheck.brute_force_prefix_split(pr["time_ns"], pr["time_bwd_ns"], pr["param_bytes"],
                                             pr["act_bytes"], 3, 4, 3, 0) == 8
    # fewer stages on more replicas: one stage ceil(10/3) + ceil(10/3) = 8; two stages best is
    # {1,2}{3,4} on (1,2) replicas: fwd max(4, 3) + bwd max(4, 3) = 8 -> ties go to the fewest stages
    assert r["opt"] == 8 and r["n_stages"] == 1 and (r["max_fwd"], r["max_bwd"]) == (4, 4)


@pytest.mark.parametrize("seed", range(8))
def test_equal_halves_reduce_to_the_min_max_search(seed):
    """Backward time = forward time: every candidate is worth twice its min-max value, so values
    double and the same candidates win in the same order; all-zero backward (or forward) times
    leave exactly the min-max search on the other half."""
    base = synth.random_small(600 + seed, 12, 6, 5, tight=[1.3, 2.0, 50.0][seed % 3], tmax=[3, 40][seed % 2])
    r0 = oracle.solve(base, keep_tables=True)
    fin = r0["V"] != INF
    for kind in ("equal", "zero_bwd", "zero_fwd"):
        pr = dict(base)
        if kind == "equal":
            pr["time_bwd_ns"] = base["time_ns"].copy()
        elif kind == "zero_bwd":
            pr["time_bwd_ns"] = np.zeros(12, np.int64)
        else:
            pr["time_bwd_ns"] = base["time_ns"].copy()
            pr["time_ns"] = np.zeros(12, np.int64)
        r = _solve(pr)
        mult = 2 if kind == "equal" else 1
        assert np.array_equal(r["V"] != INF, fin)
        assert np.array_equal(r["V"][fin], mult * r0["V"][fin])
        assert np.array_equal(r["arg_i"], r0["arg_i"]) and np.array_equal(r["arg_d"], r0["arg_d"])
        half = r["TB"] if kind != "zero_bwd" else r["TF"]
        assert np.array_equal(half[fin], r0["V"][fin])
        assert r["n_stages"] == r0["n_stages"]
        assert np.array_equal(r["stage_end"], r0["stage_end"]) and np.array_equal(r["replicas"], r0["replicas"])


@pytest.mark.parametrize("seed", range(4))
def test_single_stage_closed_form(seed):
    pr = split_case(seed, 9, 5, 1, 50.0, tmax=100)
    r = _solve(pr)
    F, Bk = int(pr["time_ns"].sum()), int(pr["time_bwd_ns"].sum())
    assert r["opt"] == defcheck.cdiv(F, 5) + defcheck.cdiv(Bk, 5) and r["n_stages"] == 1


def test_split_rejects_bad_input():
    pr = split_case(1, 5, 3, 3, 2.0)
    bad = dict(pr); bad["time_bwd_ns"] = pr["time_bwd_ns"].copy(); bad["time_bwd_ns"][1] = -3
    with pytest.raises(oracle.OracleError):
        oracle.solve(bad)
