"""Pins for the oracle's compaction step (Sec. III-B, the step that hands k blocks to the
stage-level search), on a chain.  The step is a greedy procedure, so the pins are worked examples
that follow from its sentences, invariants of any run (among them: when it stops above k groups,
no group's chosen union fits any more), and a second run of the steps written separately.  No GPU
needed."""
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


def test_worked_example_repeated_walks():
    """Eight groups of time 1, k = 1, memory not binding.  First walk: pairs {1,2} {3,4} {5,6} {7,8}
    (as above).  Second walk, all times 2, by position: {1,2} has only a right neighbour ->
    {1..4}, time 4; {3,4} is gone; {5,6} sees {1..4} (4) on the left and {7,8} (2) on the right ->
    {5..8}.  Third walk: {1..4} takes its only neighbour.  One group is left."""
    ones, zeros = np.ones(8), np.zeros(8)
    assert oracle.compact(ones, zeros, zeros, 1, 0, max_passes=1)[0].tolist() == [2, 4, 6, 8]
    assert oracle.compact(ones, zeros, zeros, 1, 0, max_passes=2)[0].tolist() == [4, 8]
    assert oracle.compact(ones, zeros, zeros, 1, 0, max_passes=3)[0].tolist() == [8]
    assert oracle.compact(ones, zeros, zeros, 1, 0)[0].tolist() == [8]
    assert oracle.compact(ones, zeros, zeros, 2, 0)[0].tolist() == [4, 8]
    # the count is checked before every merge: k = 3 is met in the middle of the second walk
    assert oracle.compact(ones, zeros, zeros, 3, 0)[0].tolist() == [4, 6, 8]


def test_worked_example_grown_group_loses_its_turn():
    """times 1 1 2 1, k = 1, one walk (groups 1, 2, 4, then 3): group 1 takes group 2; group 2 is
    gone; group 4 has only a left neighbour and joins group 3 -> {3,4}; group 3's own turn comes
    last, but the group listed under that name has grown since: no turn.  Two groups after one
    walk; the second walk merges them."""
    assert oracle.compact([1, 1, 2, 1], [0] * 4, [0] * 4, 1, 0, max_passes=1)[0].tolist() == [2, 4]
    assert oracle.compact([1, 1, 2, 1], [0] * 4, [0] * 4, 1, 0)[0].tolist() == [4]


def test_worked_example_second_walk_lists_by_current_times():
    """times 1 2 1 1 1 1, k = 2, memory not binding.  First walk (groups 1, 3, 4, 5, 6, then 2):
    group 1 takes its only neighbour -> {1,2}, time 3; group 3 sees {1,2} (3) and group 4 (1) ->
    {3,4}, time 2; group 5 sees {3,4} (2) and group 6 (1) -> {5,6}, time 2.  Second walk lists the
    groups as they now stand: {3,4} (2), {5,6} (2), {1,2} (3).  {3,4} sees {1,2} (3) on the left and
    {5,6} (2) on the right -> {3..6}.  Two groups are left.  (Listing by the times the groups had
    at the start would put {1,2} first and give {1..4}, {5,6} instead.)"""
    end, t, _, _ = oracle.compact([1, 2, 1, 1, 1, 1], [0] * 6, [0] * 6, 2, 0)
    assert end.tolist() == [2, 6] and t.tolist() == [3, 4]


def test_worked_example_walks_end_when_nothing_fits():
    """times 5 1 4 2 9 3, three bytes each, M = 9, k = 1.  First walk (list 2, 4, 6, 3, 1, 5):
    group 2 (1) takes the right neighbour (4 < 5) -> {2,3}, time 5, 6 bytes; group 4 (2) takes
    {2,3} (5 < 9) -> {2,3,4}, time 7, 9 bytes: fits exactly; group 6 takes group 5 -> {5,6}, time 12;
    group 3 is gone; group 1 (5) has only {2,3,4}: 12 bytes, refused; group 5 has grown.  Second
    walk over {1} (5), {2,3,4} (7), {5,6} (12): every chosen union needs 12 or 15 bytes: nothing is
    merged, the procedure stops at three groups."""
    end, t, p, a = oracle.compact([5, 1, 4, 2, 9, 3], [1] * 6, [2] * 6, 1, 9)
    assert end.tolist() == [1, 4, 6] and t.tolist() == [5, 7, 12] and (p + a).tolist() == [3, 9, 6]
    # one more byte of memory: in the second walk {1} (5) takes {2,3,4} (12 bytes... refused at 9, fits at 12)
    end, t, _, _ = oracle.compact([5, 1, 4, 2, 9, 3], [1] * 6, [2] * 6, 1, 12)
    assert end.tolist() == [4, 6] and t.tolist() == [12, 12]


def chosen_neighbour(tt, u):
    n = len(tt)
    if n == 1:
        return None
    if u == 0:
        return 1
    if u == n - 1:
        return n - 2
    return u + 1 if tt[u + 1] < tt[u - 1] else u - 1


@pytest.mark.parametrize("seed", range(40))
def test_invariants_and_second_run(seed):
    g = np.random.default_rng(seed)
    G = int(g.integers(1, 60))
    k = int(g.integers(1, G + 3))
    t = g.integers(0, 20, G) if seed % 2 else g.integers(0, 10**6, G)
    p, a = g.integers(0, 50, G), g.integers(0, 50, G)
    M = int(g.choice([0, 60, 150, 400, 10**9]))
    for passes in (1, 2, 0):
        end, tt, pp, aa = oracle.compact(t, p, a, k, M, max_passes=passes)
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
        if passes == 1:
            if M >= int(p.sum() + a.sum()) and k <= (G + 1) // 2:
                assert n <= max(k, (G + 1) // 2 + 1)                                   # nearly every group found a partner
        if passes == 0 and n > k:
            # stopped above k: a last walk merged nothing, so no group's chosen union fits
            for u in range(n):
                w = chosen_neighbour(tt.tolist(), u)
                assert w is None or int(pp[u] + aa[u] + pp[w] + aa[w]) > M
        if passes == 0 and M >= int(p.sum() + a.sum()):
            assert n == min(k, G)                                                      # memory never refuses: k is reached
        assert end.tolist() == defcheck.compact_steps(t, p, a, k, M, passes)


def test_walk_limit_is_a_prefix_of_the_unlimited_run():
    """n walks are the first n walks of the unlimited run: the group counts never increase with n
    and settle at the unlimited result."""
    g = np.random.default_rng(5)
    t, p, a = g.integers(0, 1000, 300), g.integers(0, 50, 300), g.integers(0, 50, 300)
    full = oracle.compact(t, p, a, 7, 900)[0]
    counts = [len(oracle.compact(t, p, a, 7, 900, max_passes=n)[0]) for n in range(1, 12)]
    assert all(x >= y for x, y in zip(counts, counts[1:])) and counts[-1] == len(full)
    assert counts[0] > counts[-1]


def test_compact_rejects_bad_input():
    with pytest.raises(oracle.OracleError):
        oracle.compact([1, -1], [0, 0], [0, 0], 1, 5)
    with pytest.raises(oracle.OracleError):
        oracle.compact([1, 2], [0, 0], [0, 0], 0, 5)
    with pytest.raises(oracle.OracleError):
        oracle.compact([1 << 61, 1 << 61], [0, 0], [0, 0], 1, 5)
