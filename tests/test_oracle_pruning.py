"""The search-space pruning printed in Algorithm 1 (trimmed loop ranges and the running bound
d_min), run as a study on the CPU oracle: what it skips and whether it changes the answer under
the additive cost model.  The HIP path does not apply it.  No GPU needed."""
import numpy as np
import pytest

import oracle
from paper_2103_16063_amd import synth

INF = oracle.INF


def both(pr, S):
    t, p, a = pr["time_ns"], pr["param_bytes"], pr["act_bytes"]
    N, D = len(t), pr["n_devices"]
    cost, fit = oracle.tables(oracle.prefix(t), oracle.prefix(p), oracle.prefix(a), D, pr["mem_capacity"])
    V, _, _ = oracle.dp(N, D, S, cost, fit)
    Vp, cells, cands, d_min = oracle.dp_pruned(N, D, S, cost, fit)
    return V, Vp, cells, cands, d_min


@pytest.mark.parametrize("seed", range(8))
def test_without_memory_pressure_only_the_ranges_are_trimmed(seed):
    """Every stage fits: d_min never moves, the value for exactly S stages is the unpruned one,
    and the numbers of visited cells and scanned candidates are those of the trimmed loops:
    level s visits b = s..N-S+s and d = s..D-S+s, a cell scans (b-s+1)(d-s+1) candidates."""
    g = np.random.default_rng(seed)
    N, D = int(g.integers(3, 30)), int(g.integers(2, 13))
    S = int(g.integers(1, min(N, D) + 1))
    pr = synth.random_small(seed, N, D, S, tight=1e6, tmax=500)
    V, Vp, cells, cands, d_min = both(pr, S)
    assert d_min == 1
    assert int(Vp[S, N, D]) == int(V[S, N, D]) != INF
    assert cells == S * (N - S + 1) * (D - S + 1)
    tri = lambda n: n * (n + 1) // 2
    assert cands == S * tri(N - S + 1) * tri(D - S + 1)
    # every visited cell holds the unpruned value
    seen = Vp != INF
    assert np.array_equal(Vp[seen], V[seen])


def test_worked_example_where_d_min_loses_the_only_plan():
    """Four blocks, four devices, exactly three stages, M = 4.  times 1 3 2 1, persistent bytes
    1 3 0 1, transient bytes 3 0 5 0.  The only plans that fit are {1}{2}{3,4} on (1,1,2) devices
    and its variants with stage {3,4} on 2 replicas (4 = 1 + ceil(5/2) bytes): slowest stage 3.
    Level 1: blocks {1,2} on 2 devices need 4 + ceil(3/2) = 6 bytes: no solution, d_min = 3.
    Level 2 therefore never tries two stages on 2 devices, the prefix the plan needs; block
    count 3 on 3 devices has no solution either (d_min = 4), and level 3 ends INFEASIBLE."""
    pr = {"name": "worked_pruning", "time_ns": np.array([1, 3, 2, 1]), "param_bytes": np.array([1, 3, 0, 1]),
          "act_bytes": np.array([3, 0, 5, 0]), "n_devices": 4, "max_stages": 3, "n_microbatches": 1,
          "mem_capacity": 4}
    V, Vp, cells, cands, d_min = both(pr, 3)
    assert int(V[3, 4, 4]) == 3
    assert int(V[2, 2, 2]) == 3 and int(Vp[2, 2, 2]) == INF   # the skipped prefix
    assert int(Vp[2, 2, 3]) == 2
    assert int(Vp[3, 4, 4]) == INF and d_min == 5
    assert cells == 3 + 2 + 1  # (1,1,2) (1,1,1) (1,2,2) | (2,2,3) (2,3,3) | (3,4,4)


def test_pruning_never_improves_and_often_hurts():
    """Pruned cells only remove candidates, so the pruned value is never below the unpruned one.
    Under this cost model it is frequently above it, or lost altogether: a single long stage that
    does not fit raises d_min for all later levels, although more stages would fit on fewer
    devices each.  That is why the search itself leaves d_min out."""
    worse = lost = total = skipped = visited = 0
    for seed in range(200):
        g = np.random.default_rng(seed)
        N, D = int(g.integers(4, 40)), int(g.integers(2, 17))
        S = int(g.integers(1, min(N, D) + 1))
        pr = synth.random_small(seed, N, D, S, tight=float(g.choice([1.1, 1.5, 2.0, 3.0, 8.0])), tmax=1000)
        V, Vp, cells, cands, d_min = both(pr, S)
        v, vp = int(V[S, N, D]), int(Vp[S, N, D])
        assert vp >= v
        total += 1
        worse += vp > v
        lost += v != INF and vp == INF
        visited += cells
        skipped += S * (N - S + 1) * (D - S + 1) - cells
    assert worse >= 20 and lost >= 3, (worse, lost, total)
    assert skipped > 0
