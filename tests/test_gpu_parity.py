"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Everything is integer, so every comparison is bit-exact."""
import numpy as np
import pytest
import torch

import oracle
from paper_2103_16063_amd import binding as B
from paper_2103_16063_amd import synth
from tests import defcheck
from tests.gpu_util import INF, assert_results_match, assert_tables_match, gpu_run, oracle_solve_many

pytestmark = pytest.mark.gpu

ALGOS = [B.ALGO_MERGE, B.ALGO_SCAN, B.ALGO_RECOMPUTE]  # RECOMPUTE acts as MERGE on 64-bit handles
WIDTHS = [B.NARROW_MAX_TOTAL_TIME, 1 << 50]


@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("width", WIDTHS)
@pytest.mark.parametrize("k", [1, 2, 3])
def test_configs_1_to_3_tables_and_plan(k, algo, width):
    pr = synth.named_config(k)
    res, sess = gpu_run([pr], algo=algo, max_total_time_ns=width)
    with sess:
        assert_results_match([pr], res)
        assert_tables_match(pr, sess, 0)


@pytest.mark.parametrize("algo", [B.ALGO_AUTO, B.ALGO_MERGE])
def test_config4_full_size(algo):
    """N=1024, D=64, S<=32 in the launch configuration the benchmark times (AUTO: stage times
    recomputed in the level kernel, the stage-time table built for the export) and with the table
    read by the level kernel (MERGE): optimum, plan, the whole value table and the whole (i, d')
    tables of every cell against the oracle (a few seconds of CPU with all cores)."""
    pr = synth.named_config(4)
    res, sess = gpu_run([pr], algo=algo)
    with sess:
        assert_results_match([pr], res)
        o = assert_tables_match(pr, sess, 0, args=True)
        t, p, a = pr["time_ns"], pr["param_bytes"], pr["act_bytes"]
        defcheck.check_plan(t, p, a, 64, 32, pr["mem_capacity"], int(res["opt"][0]),
                            int(res["n_stages"][0]), res["stage_end"][0], res["replicas"][0])
        assert o["opt"] == 5541252 and o["n_stages"] == 12


SHAPES = [  # (N, D, S): edge shapes, ragged tails, several 64-column chunks, non-power-of-two D
    (1, 1, 1), (1, 7, 3), (9, 1, 4), (3, 3, 9), (2, 64, 2), (5, 2, 5),
    (16, 4, 4), (33, 5, 5), (63, 8, 8), (64, 9, 6), (65, 12, 7), (100, 17, 9),
    (129, 24, 6), (130, 33, 5), (200, 40, 4), (70, 63, 10), (96, 64, 12),
    (64, 64, 64), (80, 64, 64), (65, 33, 40),  # as many levels as devices
]


@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("width", WIDTHS)
def test_shape_sweep_single(algo, width):
    for n, (N, D, S) in enumerate(SHAPES):
        for tight in (1.05, 1.6, 40.0):
            pr = synth.random_small(900 + n, N, D, S, tight=tight, tmax=5000)
            if width > B.NARROW_MAX_TOTAL_TIME:
                pr["time_ns"] = pr["time_ns"] * (1 << 24)  # totals beyond 32 bits
            res, sess = gpu_run([pr], algo=algo, max_total_time_ns=width)
            with sess:
                assert_results_match([pr], res)
                assert_tables_match(pr, sess, 0, args=(N <= 100))


@pytest.mark.parametrize("algo", ALGOS)
def test_ties_and_zero_times(algo):
    """Constant and zero block times: many equal candidates per cell, so the smallest-(i,d')
    rule and the smallest-s rule decide the plan."""
    for seed in range(6):
        N, D, S = 40, 9, 6
        pr = synth.random_small(300 + seed, N, D, S, tight=[1.2, 2.0, 50.0][seed % 3], tmax=3,
                                zero_time_frac=0.3)
        if seed >= 3:
            pr["time_ns"] = np.full(N, seed - 3, dtype=np.int64)  # includes all-zero times
        res, sess = gpu_run([pr], algo=algo)
        with sess:
            assert_results_match([pr], res)
            assert_tables_match(pr, sess, 0)


def test_infeasible_and_oversized_block():
    pr = synth.random_small(1, 30, 6, 5, tight=5.0)
    pr["param_bytes"] = pr["param_bytes"].copy()
    pr["param_bytes"][11] = pr["mem_capacity"] + 1
    pr2 = synth.random_small(2, 20, 4, 4, tight=0.3)  # capacity far too small
    res, sess = gpu_run([pr, pr2])
    with sess:
        assert (res["opt"] == INF).all() and (res["n_stages"] == 0).all()
        assert (res["stage_end"] == -1).all() and (res["replicas"] == -1).all()
        assert (res["est_iter_ns"] == INF).all()
        assert_results_match([pr, pr2], res)
        assert_tables_match(pr, sess, 0)


@pytest.mark.parametrize("algo", ALGOS)
def test_batched_mixed_shapes(algo):
    """One launch sequence over problems of different N, D, S, MB and capacity: each equals
    its oracle solve and its own single-problem GPU solve, byte for byte."""
    g = np.random.default_rng(7)
    probs = []
    for q in range(40):
        N = int(g.integers(1, 150))
        D = int(g.choice([1, 2, 3, 5, 8, 9, 16, 17, 31, 32, 33, 48, 64]))
        S = int(g.integers(1, 12))
        probs.append(synth.random_small(2000 + q, N, D, S, tight=float(g.choice([0.9, 1.3, 2.0, 30.0])),
                                        tmax=int(g.choice([3, 100, 100000]))))
    res, sess = gpu_run(probs, algo=algo)
    with sess:
        assert_results_match(probs, res)
        for q in (0, 7, 19, 39):
            assert_tables_match(probs[q], sess, q, args=(probs[q]["time_ns"].shape[0] <= 100))
    for q in (3, 11, 25):
        r1, s1 = gpu_run([probs[q]], algo=algo)
        with s1:
            for key in ("opt", "n_stages", "est_iter_ns"):
                assert r1[key][0] == res[key][q]
            k = r1["stage_end"].shape[1]
            assert np.array_equal(r1["stage_end"][0], res["stage_end"][q][:k])
            assert np.array_equal(r1["replicas"][0], res["replicas"][q][:k])


_C5_ORACLE = []


@pytest.mark.parametrize("algo", [B.ALGO_AUTO, B.ALGO_MERGE])
def test_config5_batched_sweep_full_size(algo):
    """All 2048 searches in one batch, in the launch configuration the benchmark times (AUTO) and
    with the stage-time tables read by the level kernels (MERGE).  The oracle solves every one of
    them (one search per host thread): optimum, stage count, estimated iteration time and the
    canonical plan must agree for all 2048; the tables of a few are compared cell by cell; every
    plan is also checked from the definition."""
    probs = synth.named_config(5)
    if not _C5_ORACLE:
        _C5_ORACLE.extend(oracle_solve_many(probs))
    res, sess = gpu_run(probs, algo=algo)
    with sess:
        assert (res["status"] == 0).all()
        assert_results_match(probs, res, oracle_results=_C5_ORACLE)
        for q in (0, 1, 2, 3, 1000, 2047):  # covers the four device-count classes
            assert_tables_match(probs[q], sess, q, args=False)
        assert {probs[q]["n_devices"] for q in (0, 1, 2, 3, 1000, 2047)} == {8, 16, 32, 64}
        for q, pr in enumerate(probs):
            D = pr["n_devices"]
            opt, ns = int(res["opt"][q]), int(res["n_stages"][q])
            defcheck.check_plan(pr["time_ns"], pr["param_bytes"], pr["act_bytes"], D, 16,
                                pr["mem_capacity"], opt, ns, res["stage_end"][q], res["replicas"][q])
        assert (res["opt"] != INF).sum() > 1500


def test_deterministic_across_runs():
    probs = synth.batched_sweep(Q=64)
    res1, s1 = gpu_run(probs)
    with s1:
        V1 = s1.table(B.TABLE_V, 5)
        s1.solve()
        s1.traceback()
        res2 = s1.run()
        V2 = s1.table(B.TABLE_V, 5)
    for k in res1:
        assert np.array_equal(res1[k], res2[k]), k
    assert np.array_equal(V1, V2)


def test_merge_recompute_and_scan_levels_agree_at_medium_size():
    pr = synth.enlarged_transformer_chain(seed=11, N=300, D=48, S=20, M=24 * synth.GiB)
    rm, sm = gpu_run([pr], algo=B.ALGO_MERGE)
    rs, ss = gpu_run([pr], algo=B.ALGO_SCAN)
    rr, sr = gpu_run([pr], algo=B.ALGO_RECOMPUTE)
    with sm, ss, sr:
        assert np.array_equal(sm.table(B.TABLE_V, 0), ss.table(B.TABLE_V, 0))
        assert np.array_equal(sm.table(B.TABLE_V, 0), sr.table(B.TABLE_V, 0))
        assert np.array_equal(sm.table(B.TABLE_COST, 0), sr.table(B.TABLE_COST, 0))  # built for the export
        for k in rm:
            assert np.array_equal(rm[k], rs[k]), k
            assert np.array_equal(rm[k], rr[k]), k
        assert_results_match([pr], rm)


def test_recomputed_stage_times_at_the_edges_of_the_value_range():
    """The level kernel that recomputes ceil(T / r) without an integer division, on totals that sit
    at exact multiples of r, one above and one below them, at the top of the 32-bit range, and at
    0: every stage time it forms is one the table builder forms too, so the value tables of the two
    level kernels must be identical (and equal the oracle's)."""
    g = np.random.default_rng(4242)
    probs = []
    for case in range(24):
        N = int(g.integers(40, 129))
        D = int(g.choice([7, 8, 16, 31, 32, 33, 63, 64]))
        pr = synth.random_small(9100 + case, N, D, int(g.integers(2, 14)), tight=float(g.choice([1.3, 3.0, 60.0])), tmax=9)
        kind = case % 4
        if kind == 0:      # stage totals are multiples of 720720 = lcm(1..16): exact quotients for many r
            pr["time_ns"] = np.full(N, 720720, dtype=np.int64) * g.integers(0, 3, N)
        elif kind == 1:    # one off the multiples
            pr["time_ns"] = np.full(N, 720720, dtype=np.int64) * g.integers(0, 3, N) + g.integers(-1, 2, N) * (g.random(N) < 0.2)
            pr["time_ns"] = np.maximum(pr["time_ns"], 0)
        elif kind == 2:    # the whole chain just fits the 32-bit range
            t = g.integers(0, 1 << 20, N).astype(np.int64)
            t[int(g.integers(0, N))] += (B.NARROW_MAX_TOTAL_TIME - int(t.sum()))
            pr["time_ns"] = t
        else:              # powers of two and their neighbours
            pr["time_ns"] = (1 << g.integers(0, 24, N)).astype(np.int64) + g.integers(-1, 2, N)
        probs.append(pr)
    rm, sm = gpu_run(probs, algo=B.ALGO_MERGE)
    rr, sr = gpu_run(probs, algo=B.ALGO_RECOMPUTE, one_launch_small=1)
    ro, so = gpu_run(probs, algo=B.ALGO_RECOMPUTE, one_launch_small=2)   # the one-launch kernel's own recomputation
    with sm, sr, so:
        rc, info = B.rannc_dp_solve_info(so.h)
        assert [info.level_kernel[k] for k in range(3)] == [B.KERNEL_ONE_LAUNCH_RECOMPUTE] * 3
        for k in rm:
            assert np.array_equal(rm[k], rr[k]), k
            assert np.array_equal(rm[k], ro[k]), k
        assert (rm["status"] == 0).all()
        for q in range(len(probs)):
            assert np.array_equal(sm.table(B.TABLE_V, q), sr.table(B.TABLE_V, q)), q
            assert np.array_equal(sm.table(B.TABLE_V, q), so.table(B.TABLE_V, q)), q
        assert_results_match(probs, rr)
        for q in (0, 1, 2, 3, 5, 10, 15, 20):   # every kind of total; the table builder divides the same way
            assert_tables_match(probs[q], sr, q, args=False)
            assert_tables_match(probs[q], sm, q, args=False)


def test_recomputed_stage_times_64_bit_values_at_the_edges_of_their_range():
    """The one-launch kernel's recomputation on 64-bit values is exact for stage times up to 2^40 ns
    (the handle's bound says so).  Chains whose total is exactly 2^40, whose stage totals are
    multiples of many r at once (and one off them) far above the 32-bit range, and powers of two
    with their neighbours: identical tables with the stage times read from the table on a handle
    of a larger bound, and equal to the oracle's."""
    g = np.random.default_rng(777)
    top = B.WIDE_RECOMPUTE_MAX_TOTAL_TIME
    probs = []
    for case in range(24):
        N = int(g.integers(20, 129))
        D = int(g.choice([7, 8, 16, 31, 32]))
        pr = synth.random_small(9300 + case, N, D, int(g.integers(2, 14)), tight=float(g.choice([1.3, 3.0, 60.0])), tmax=9)
        kind = case % 4
        unit = 720720 * 11 * 13 * 17   # lcm(1..17) * ... : exact quotients for many r, about 2^31
        if kind == 0:
            pr["time_ns"] = np.full(N, unit, dtype=np.int64) * g.integers(0, 3, N)
        elif kind == 1:
            pr["time_ns"] = np.maximum(np.full(N, unit, dtype=np.int64) * g.integers(0, 3, N)
                                       + g.integers(-1, 2, N) * (g.random(N) < 0.2), 0)
        elif kind == 2:    # the whole chain is exactly the bound
            t = g.integers(0, 1 << 32, N).astype(np.int64)
            t[int(g.integers(0, N))] += top - int(t.sum())
            pr["time_ns"] = t
        else:
            pr["time_ns"] = (1 << g.integers(0, 33, N)).astype(np.int64) + g.integers(-1, 2, N)
        assert 0 <= int(pr["time_ns"].min()) and int(pr["time_ns"].sum()) <= top
        probs.append(pr)
    rt, st = gpu_run(probs, max_total_time_ns=1 << 50, one_launch_small=1)
    ro, so = gpu_run(probs, max_total_time_ns=top, one_launch_small=2)
    with st, so:
        rc, info = B.rannc_dp_solve_info(so.h)
        assert [info.level_kernel[k] for k in range(3)] == [B.KERNEL_ONE_LAUNCH_RECOMPUTE] * 3
        rc, info = B.rannc_dp_solve_info(st.h)
        assert B.KERNEL_ONE_LAUNCH_RECOMPUTE not in [info.level_kernel[k] for k in range(3)]
        assert (rt["status"] == 0).all()
        for k in rt:
            assert np.array_equal(rt[k], ro[k]), k
        for q in range(len(probs)):
            assert np.array_equal(st.table(B.TABLE_V, q), so.table(B.TABLE_V, q)), q
        assert_results_match(probs, ro)
        for q in (0, 1, 2, 3, 6, 11, 18, 23):
            assert_tables_match(probs[q], so, q, args=False)


@pytest.mark.parametrize("algo", [B.ALGO_MERGE, B.ALGO_RECOMPUTE])
@pytest.mark.parametrize("rows", [1, 2, 4, 8, 12, 16])
def test_rows_per_wave_variants(rows, algo):
    """A wave of the merge level kernel takes 1, 2, 4, 8, 12 or 16 predecessor rows one after the other
    (work items of 4 to 64 rows); the handle's limits fix the choice.  All must give the
    oracle's tables, with the stage times read from their table and recomputed."""
    probs = [synth.enlarged_transformer_chain(seed=21, N=333, D=64, S=12, M=24 * synth.GiB),
             synth.random_small(77, 150, 40, 9, tight=1.3, tmax=5000),
             synth.random_small(78, 65, 7, 7, tight=1.1, tmax=50)]
    for width in WIDTHS:
        res, sess = gpu_run(probs, max_total_time_ns=width, rows_per_wave=rows, algo=algo, one_launch_small=1)
        with sess:
            rc, info = B.rannc_dp_solve_info(sess.h)
            want = B.KERNEL_MERGE_RECOMPUTE if (algo == B.ALGO_RECOMPUTE and width == B.NARROW_MAX_TOTAL_TIME) \
                else B.KERNEL_MERGE_TABLE
            assert rc == B.OK and list(info.n_problems) == [1, 0, 0, 2]
            assert [info.level_kernel[k] for k in (0, 3)] == [want, want]
            assert_results_match(probs, res)
            for q in range(3):
                assert_tables_match(probs[q], sess, q, args=False)


@pytest.mark.parametrize("width", WIDTHS)
def test_random_batches_against_oracle(width):
    """Several hundred random searches (chains of 1..200 blocks, every device count 1..64, tight
    and loose memory, small value ranges that force ties) in batches of 64."""
    g = np.random.default_rng(12345)
    for batch in range(4):
        probs = []
        for q in range(64):
            N = int(g.integers(1, 200))
            D = int(g.integers(1, 65))
            S = int(g.integers(1, 20))
            pr = synth.random_small(7000 + 64 * batch + q, N, D, S,
                                    tight=float(g.choice([0.8, 1.0, 1.2, 1.6, 3.0, 100.0])),
                                    tmax=int(g.choice([1, 4, 1000, 10 ** 6])),
                                    zero_time_frac=float(g.choice([0.0, 0.0, 0.3])))
            if width > B.NARROW_MAX_TOTAL_TIME and q % 2:
                pr["time_ns"] = pr["time_ns"] * (1 << 22)
            probs.append(pr)
        res, sess = gpu_run(probs, max_total_time_ns=width)
        with sess:
            assert_results_match(probs, res)
            for q in (0, 13, 37, 63):
                assert_tables_match(probs[q], sess, q, args=(probs[q]["time_ns"].shape[0] <= 80))


@pytest.mark.parametrize("width", WIDTHS)
def test_plan_recovery_from_lds_and_from_memory(width):
    """Plan recovery of a launch of at most 64 small searches first copies what the walk reads into
    LDS; larger launches, and searches whose tables do not fit, walk through memory.  The same
    searches alone, in a batch of 30 and inside a batch of 72: identical plans, all equal to the
    oracle's, also for a forced exact stage count."""
    g = np.random.default_rng(77)
    probs = []
    for q in range(30):
        N = int(g.integers(2, 100))
        D = int(g.choice([3, 8, 12, 16, 25, 32, 40, 64]))
        probs.append(synth.random_small(7000 + q, N, D, int(g.integers(2, 20)), tight=float(g.choice([1.3, 2.5, 40.0])),
                                        tmax=int(g.choice([5, 10 ** 5]))))
        if width > B.NARROW_MAX_TOTAL_TIME:
            probs[-1]["time_ns"] = probs[-1]["time_ns"] * (1 << 22)
    more = [synth.random_small(7100 + q, 20, 8, 4, tight=2.0) for q in range(42)]
    r30, s30 = gpu_run(probs, max_total_time_ns=width)
    r72, s72 = gpu_run(probs + more, max_total_time_ns=width)
    with s30, s72:
        assert_results_match(probs, r30)
        for k in r30:
            assert np.array_equal(r30[k], r72[k][:30]), k
    r1, s1 = gpu_run(probs[:1], max_total_time_ns=width)
    with s1:
        for k in r1:
            if r1[k].ndim == 2:   # plan arrays: the stride is the batch's largest stage count
                w = r1[k].shape[1]
                assert np.array_equal(r1[k], r30[k][:1, :w]) and (r30[k][:1, w:] == -1).all(), k
            else:
                assert np.array_equal(r1[k], r30[k][:1]), k


@pytest.mark.parametrize("algo", [B.ALGO_AUTO, B.ALGO_MERGE])
@pytest.mark.parametrize("mode", [1, 2])
@pytest.mark.parametrize("width", [B.NARROW_MAX_TOTAL_TIME, B.WIDE_RECOMPUTE_MAX_TOTAL_TIME, 1 << 50])
def test_small_search_kernel_on_and_off(mode, width, algo):
    """Searches of at most 128 blocks can run as one launch with one workgroup per search (levels
    folded in LDS) or through the per-level launches; the library chooses by batch shape.  Both
    are forced here (1 = never, 2 = always) on the same inputs: identical tables, optimum, plan.
    The one-launch kernel recomputes the stage times (up to the 32-device class, 32-bit values or
    64-bit values on a handle whose time bound is at most 2^40 ns, unless the handle asks for the
    table) or reads them from the table it builds: all of these run here."""
    g = np.random.default_rng(99)
    probs = [synth.named_config(1), synth.named_config(2)]
    for q in range(30):
        N = int(g.integers(1, 129))
        D = int(g.choice([1, 2, 4, 7, 8, 9, 16, 17, 32, 33, 64]))
        probs.append(synth.random_small(4000 + q, N, D, int(g.integers(1, 18)),
                                        tight=float(g.choice([0.9, 1.2, 2.0, 50.0])),
                                        tmax=int(g.choice([2, 1000, 10 ** 6])),
                                        zero_time_frac=float(g.choice([0.0, 0.25]))))
    res, sess = gpu_run(probs, max_total_time_ns=width, one_launch_small=mode, algo=algo)
    with sess:
        rc, info = B.rannc_dp_solve_info(sess.h)
        assert rc == B.OK and all(info.n_problems[k] for k in range(4))
        kinds = [info.level_kernel[k] for k in range(4)]
        if mode == 2:
            recomputes = width <= B.WIDE_RECOMPUTE_MAX_TOTAL_TIME and algo == B.ALGO_AUTO
            assert kinds == ([B.KERNEL_ONE_LAUNCH_RECOMPUTE] * 3 if recomputes else [B.KERNEL_ONE_LAUNCH] * 3) + [B.KERNEL_ONE_LAUNCH]
        else:
            assert not {B.KERNEL_ONE_LAUNCH, B.KERNEL_ONE_LAUNCH_RECOMPUTE} & set(kinds)
        assert_results_match(probs, res)
        for q in range(0, len(probs), 3):
            assert_tables_match(probs[q], sess, q, args=(probs[q]["time_ns"].shape[0] <= 100))


@pytest.mark.parametrize("width", [B.NARROW_MAX_TOTAL_TIME, B.WIDE_RECOMPUTE_MAX_TOTAL_TIME])
def test_one_launch_recompute_block_shapes(width):
    """The recomputing one-launch kernel packs row pairs of the triangular blocks and short rows of
    the rectangular block into passes of 64 lanes; the packing depends on the widths min(64, N) and
    N - 64.  Every kind of width (one column, odd, a power of two, one more or less than one, the
    full 64) in both chunks, at 8 and 32 devices: tables, optimum and plan against the oracle."""
    probs = []
    for q, N in enumerate([1, 2, 3, 5, 8, 15, 16, 17, 31, 32, 33, 47, 63, 64, 65, 66, 67, 72, 80, 81,
                           95, 96, 97, 111, 127, 128]):
        for D in (8, 32):
            probs.append(synth.random_small(7000 + 2 * q + (D == 32), N, D, min(D, 12),
                                            tight=1.2 if q % 3 else 50.0, tmax=10 ** 6,
                                            zero_time_frac=0.25 if q % 4 == 0 else 0.0))
    res, sess = gpu_run(probs, one_launch_small=2, max_total_time_ns=width)
    with sess:
        rc, info = B.rannc_dp_solve_info(sess.h)
        assert rc == B.OK
        assert [info.level_kernel[k] for k in range(4) if info.n_problems[k]] == [B.KERNEL_ONE_LAUNCH_RECOMPUTE] * 2
        assert_results_match(probs, res)
        for q in range(len(probs)):
            assert_tables_match(probs[q], sess, q, args=False)


@pytest.mark.parametrize("N,M_gib,width", [(4096, 64, B.NARROW_MAX_TOTAL_TIME), (3000, 48, 1 << 50)])
def test_large_search_prefix_parity_and_properties(N, M_gib, width):
    """A search four times config 4's length (64 column chunks, a ragged one at N = 3000, 2 GB of
    table), beyond what the oracle finishes in seconds.  The values of a prefix of the chain do not
    depend on the blocks behind it, so the cells with j <= 192 are compared one by one with the
    oracle's run on the first 192 blocks; the rest is checked by what holds at any size: the plan
    is valid and attains the optimum, the optimum is at least the perfectly balanced time, and
    the values do not increase with the device total."""
    pr = synth.enlarged_transformer_chain(seed=11, N=N, D=64, S=32, MB=64, M=M_gib << 30)
    res, sess = gpu_run([pr], max_total_time_ns=width)
    with sess:
        opt, ns = int(res["opt"][0]), int(res["n_stages"][0])
        assert int(res["status"][0]) == 0 and opt != INF and 1 <= ns <= 32
        t, p, a = pr["time_ns"], pr["param_bytes"], pr["act_bytes"]
        defcheck.check_plan(t, p, a, 64, 32, pr["mem_capacity"], opt, ns, res["stage_end"][0], res["replicas"][0])
        assert opt >= -(-int(t.sum()) // 64)
        V = sess.table(B.TABLE_V, 0)
        J = 192
        head = dict(pr)
        for k in ("time_ns", "param_bytes", "act_bytes"):
            head[k] = pr[k][:J]
        o = oracle.solve(head, n_threads=0, keep_tables=True)
        assert np.array_equal(V[:, :J + 1, :], o["V"])
        fin = V[1:, 1:, 1:]
        assert (fin[:, :, 1:] <= fin[:, :, :-1]).all()          # non-increasing in d
        col = V[1:, N, 64]
        assert opt == int(col.min()) and ns == 1 + int(np.argmin(col))
        # the plan of an exact stage count further down the column is valid too
        s_other = ns + 3
        assert int(V[s_other, N, 64]) != INF
        lev = torch.full((1,), s_other, dtype=torch.int32, device="cuda:0")
        assert B.rannc_dp_traceback_at(sess.h, sess.stream(), lev, sess.plan_stride, sess.d_se, sess.d_rp) == B.OK
        torch.cuda.synchronize()
        defcheck.check_plan(t, p, a, 64, 32, pr["mem_capacity"], int(V[s_other, N, 64]), s_other,
                            sess.d_se.cpu().numpy()[0], sess.d_rp.cpu().numpy()[0])


@pytest.mark.parametrize("single_stream", [0, 1])
@pytest.mark.parametrize("timing", [False, True])
def test_classes_on_their_own_streams(single_stream, timing):
    """A batch with all four device-count classes: the classes run as independent chains of
    launches on streams of the handle (the default) or one after the other on the caller's stream
    (limits.single_stream = 1, and whenever per-phase timing is on).  Same results either way, also
    on repeated solves of one handle and with the one-launch kernel on or off."""
    probs = []
    for seed in range(64):
        g = np.random.default_rng(121_000 + seed)
        D = int(g.choice([3, 8, 11, 16, 27, 32, 50, 64]))
        probs.append(synth.random_small(seed, int(g.integers(1, 140)), D, int(g.integers(1, 18)),
                                        tight=float(g.choice([1.2, 2.0, 9.0])), tmax=int(g.choice([9, 4000]))))
    for fused in (1, 0):
        res, sess = gpu_run(probs, single_stream=single_stream, one_launch_small=fused)
        with sess:
            B.rannc_dp_set_timing(sess.h, timing)
            for _ in range(3):
                again = sess.run()
                for k in res:
                    assert np.array_equal(res[k], again[k]), k
            assert_results_match(probs, res)
            assert_tables_match(probs[7], sess, 7, args=False)


def test_solve_on_a_side_stream_and_two_handles_at_once():
    """The caller's stream is a stream of its own (not the default one), and two handles work at
    the same time on two such streams; each batch has several device-count classes, so each
    handle also forks to its own streams and joins back."""
    batches = []
    for b in range(2):
        probs = []
        for seed in range(40):
            g = np.random.default_rng(131_000 + 100 * b + seed)
            probs.append(synth.random_small(seed + 100 * b, int(g.integers(1, 150)), int(g.integers(1, 65)),
                                            int(g.integers(1, 14)), tight=float(g.choice([1.3, 3.0])), tmax=2000))
        batches.append(probs)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    sessions = [B.Session(synth.concat_batch(p)) for p in batches]
    try:
        torch.cuda.synchronize()
        for rep in range(3):
            for sess, st in zip(sessions, streams):
                with torch.cuda.stream(st):
                    sess.solve()
                    sess.traceback()
        outs = []
        for sess, st in zip(sessions, streams):
            with torch.cuda.stream(st):
                outs.append(sess.run())
        for probs, res in zip(batches, outs):
            assert_results_match(probs, res)
    finally:
        for sess in sessions:
            sess.close()


@pytest.mark.parametrize("fused", [1, 2])
def test_more_searches_than_one_grid_dimension_holds(fused):
    """70 000 searches in one batch (a launch covers at most 65 535 problems in a grid dimension, so
    every kernel is launched in slices): seven distinct tiny searches, each repeated 10 000 times;
    every copy must equal the oracle's result for its original."""
    base = [synth.random_small(4000 + k, 2 + k, 1 + (k * 5) % 9, 1 + k % 4, tight=[1.2, 2.0, 9.0][k % 3], tmax=50)
            for k in range(7)]
    probs = [base[q % 7] for q in range(70_000)]
    res, sess = gpu_run(probs, one_launch_small=fused)
    with sess:
        for k, pr in enumerate(base):
            o = oracle.solve(pr)
            sel = slice(k, None, 7)
            assert (res["status"][sel] == 0).all()
            assert (res["opt"][sel] == o["opt"]).all() and (res["n_stages"][sel] == o["n_stages"]).all()
            assert (res["est_iter_ns"][sel] == o["est_iter_ns"]).all()
            w = min(res["stage_end"].shape[1], len(o["stage_end"]))
            assert (res["stage_end"][sel, :w] == o["stage_end"][:w]).all()
            assert (res["replicas"][sel, :w] == o["replicas"][:w]).all()
            assert (res["stage_end"][sel, w:] == -1).all()


def test_environment_overrides_and_automatic_choice_of_the_level_kernel(monkeypatch):
    """What rannc_dp_solve_info reports: a large class of a 32-bit batch has its stage times
    recomputed, a small one reads the table, 64-bit handles and batches with a communication term
    always read the table; the documented environment variables override the limits' tuning."""
    big = synth.batched_sweep(Q=1000)
    big = [p for p in big if p["n_devices"] == 64][:200] + [p for p in big if p["n_devices"] == 32][:2]
    res, sess = gpu_run(big)
    with sess:
        rc, info = B.rannc_dp_solve_info(sess.h)
        assert rc == B.OK and list(info.n_problems) == [0, 0, 2, 200]
        assert info.level_kernel[3] == B.KERNEL_MERGE_RECOMPUTE and info.level_kernel[2] == B.KERNEL_MERGE_TABLE
        assert_results_match(big[:6] + big[-2:], {k: np.concatenate([v[:6], v[-2:]]) for k, v in res.items()})
    res, sess = gpu_run(big, max_total_time_ns=1 << 50)
    with sess:
        rc, info = B.rannc_dp_solve_info(sess.h)
        assert [info.level_kernel[k] for k in (2, 3)] == [B.KERNEL_MERGE_TABLE] * 2
    comm = [synth.with_cut_bytes(p, 5, 100_000) for p in big]
    res, sess = gpu_run(comm, algo=B.ALGO_RECOMPUTE)
    with sess:
        rc, info = B.rannc_dp_solve_info(sess.h)
        assert [info.level_kernel[k] for k in (2, 3)] == [B.KERNEL_MERGE_TABLE] * 2
        assert_results_match(comm[:3], {k: v[:3] for k, v in res.items()})
    small = [synth.random_small(5, 40, 8, 4, tight=2.0), synth.random_small(6, 90, 30, 6, tight=2.0)]
    monkeypatch.setenv("RANNC_DP_FUSED_SMALL", "2")
    monkeypatch.setenv("RANNC_DP_ROWS_PER_WAVE", "2")
    monkeypatch.setenv("RANNC_DP_STREAMS", "0")
    res, sess = gpu_run(small, one_launch_small=1)
    with sess:
        rc, info = B.rannc_dp_solve_info(sess.h)
        assert [info.level_kernel[k] for k in (0, 2)] == [B.KERNEL_ONE_LAUNCH_RECOMPUTE] * 2
        assert_results_match(small, res)
