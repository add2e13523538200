"""Pins for the oracle's compaction step (Sec. III-B, the step that hands k blocks to the
stage-level search), on a chain.  The step is a greedy procedure, so the pins are worked examples
that follow from its sentences, invariants of any run, and a second run of the steps written
separately.  No GPU needed."""
import numpy as np
import pytest

import oracle
from tests import defcheck


def test_worked_example_distinct_times():
    """times 5 1 4 2 9 3, k = 3, memory not binding.  Listed by time: groups 2, 4, 6, 3, 1, 5.
    Group 2 (time 1) has neighbours of time 5 and 4: takes the right one -> {2,3}, time 5.
    Group 4 (time 2) has {2,3} (5) on the left and group 5 (9) on the right: left -> {2,3,4}, time 7.
    Group 6 (time 3) has only a left neighbour -> {5,6}, time 12.  Three groups are left: stop."""
    end, t, p, a = oracle.compact([5, 1, 4, 2, 9, 3], [1] * 6, [2] * 6, 3, 10**9)
    assert end.tolist() == [1, 4, 6] and t.tolist() == [5, 7, 12]
    assert p.tolist() == [1, 3, 2] and a.tolist() == [2, 6, 4]


def test_worked_example_equal_times_pair_up():
    """Eight groups of time 1, k = 4: group 1 has only a right neighbour -> {1,2}; group 2 is gone;
    group 3 sees {1,2} (2) on the left and group 4 (1) on the right -> {3,4}; likewise {5,6}, {7,8}."""
    end, t, _, _ = oracle.compact(np.ones(8), np.zeros(8), np.zeros(8), 4, 0)
    assert end.tolist() == [2, 4, 6, 8] and t.tolist() == [2, 2, 2, 2]
    # equal neighbours: the left one is taken
    end, _, _, _ = oracle.compact([3, 1, 3], [0] * 3, [0] * 3, 2, 0)
    assert end.tolist() == [2, 3]


def test_memory_rule_and_no_second_choice():
    """The chosen neighbour is the one with the smaller time; if that union does not fit, the
    other neighbour is not tried.  Bytes 6 | 1 | 1 with M = 7: group 2 (time 1) prefers the left
    neighbour (time 2 < 5), whose union needs 7 bytes: fits exactly (only more than M is refused).
    With M = 6 it is refused, although the right union (2 bytes) would fit."""
    t, p, a = [2, 1, 5], [3, 1, 1], [3, 0, 0]
    assert oracle.compact(t, p, a, 2, 7)[0].tolist() == [2, 3]
    # with M = 6: group 2 refused; group 1 (time 2) then tries its only neighbour: 7 > 6 refused;
    # group 3 (time 5) takes its only neighbour, group 2: 2 bytes fit
    assert oracle.compact(t, p, a, 2, 6)[0].tolist() == [1, 3]
    assert oracle.compact(t, p, a, 2, 1)[0].tolist() == [1, 2, 3]


@pytest.mark.parametrize("seed", range(40))
def test_invariants_and_second_run(seed):
    g = np.random.default_rng(seed)
    G = int(g.integers(1, 60))
    k = int(g.integers(1, G + 3))
    t = g.integers(0, 20, G) if seed % 2 else g.integers(0, 10**6, G)
    p, a = g.integers(0, 50, G), g.integers(0, 50, G)
    M = int(g.choice([0, 60, 150, 400, 10**9]))
    end, tt, pp, aa = oracle.compact(t, p, a, k, M)
    n = len(end)
    assert end[-1] == G and (np.diff(np.concatenate(([0], end))) >= 1).all()      # contiguous cover
    assert int(tt.sum()) == int(t.sum()) and int(pp.sum()) == int(p.sum()) and int(aa.sum()) == int(a.sum())
    assert n >= min(k, G) and n <= G
    if G <= k:
        assert n == G                                                              # nothing to do
    sizes = np.diff(np.concatenate(([0], end)))
    for u in range(n):
        if sizes[u] > 1:
            assert int(pp[u] + aa[u]) <= M                                         # every union fits
    assert G - n <= (G + 1) // 2 + G // 2                                          # a pass: one try per listed group
    if M >= int(p.sum() + a.sum()) and k <= (G + 1) // 2:
        assert n <= max(k, (G + 1) // 2 + 1)                                       # nearly every group found a partner
    assert end.tolist() == defcheck.compact_steps(t, p, a, k, M)


def test_compact_rejects_bad_input():
    with pytest.raises(oracle.OracleError):
        oracle.compact([1, -1], [0, 0], [0, 0], 1, 5)
    with pytest.raises(oracle.OracleError):
        oracle.compact([1, 2], [0, 0], [0, 0], 0, 5)
    with pytest.raises(oracle.OracleError):
        oracle.compact([1 << 61, 1 << 61], [0, 0], [0, 0], 1, 5)
