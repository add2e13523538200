"""GPU parity on random batches with the options of the search drawn together: send times on or
off, split objective on or off, 32-bit / packed 64-bit / full 64-bit handles, merge or literal level
kernel, one-launch kernel forced on / off / by rule, work items of the level kernel of a fixed size or
by rule, device-count classes on one stream or several.
Every problem against the oracle (optimum, stage count, canonical plan); one small problem per
batch also table by table.  Integers: bit-exact."""
import os

import numpy as np
import pytest

from paper_2103_16063_amd import binding as B
from paper_2103_16063_amd import synth
from tests.gpu_util import assert_results_match, assert_tables_match, gpu_run

pytestmark = pytest.mark.gpu
KNOBS = ("RANNC_DP_FUSED_SMALL", "RANNC_DP_STREAMS")


def _random_batch(g):
    comm, split = bool(g.integers(0, 2)), bool(g.integers(0, 3) == 0)
    probs = []
    for _ in range(int(g.integers(1, 14))):
        N = int(g.choice([1, 2, 3, 7, 16, 31, 33, 63, 64, 65, 96, 127, 128, 129, 150, 200]))
        D = int(g.choice([1, 2, 3, 5, 8, 9, 16, 17, 24, 32, 33, 48, 63, 64]))
        S = int(g.choice([1, 2, 3, 4, 8, 16, 40]))
        if N * N * D * D * min(S, N, D) > 4e9:
            N = 64  # keeps the oracle to a fraction of a second
        tmax = int(g.choice([3, 50, 1000, 10**6]))  # 3: ties everywhere
        pr = synth.random_small(int(g.integers(0, 1 << 30)), N, D, S,
                                tight=float(g.choice([0.6, 0.9, 1.1, 1.5, 2.5, 8.0])), tmax=tmax,
                                zero_time_frac=float(g.choice([0.0, 0.3])), zero_act=bool(g.integers(0, 5) == 0))
        if comm:
            pr = synth.with_cut_bytes(pr, int(g.integers(0, 1 << 30)), int(g.choice([1, 1000, 25_000])), lo=0,
                                      hi=int(g.choice([10, 1 << 20])), zero_frac=float(g.choice([0.0, 0.5])))
        if split:
            pr = synth.with_backward_times(pr, int(g.integers(0, 1 << 30)), tmax=int(g.choice([0, 5, tmax])))
        probs.append(pr)
    return probs


@pytest.mark.parametrize("group", range(8))
def test_random_batches_with_mixed_options(group):
    saved = {k: os.environ.get(k) for k in KNOBS}
    try:
        for rnd in range(25):
            g = np.random.default_rng(910_000 + 100 * group + rnd)
            width = [B.NARROW_MAX_TOTAL_TIME, 1 << 40, 1 << 50][int(g.integers(0, 3))]
            algo = B.ALGO_SCAN if g.integers(0, 6) == 0 else B.ALGO_AUTO
            for k, v in zip(KNOBS, (["", "0", "2"][int(g.integers(0, 3))], ["", "0"][int(g.integers(0, 2))])):
                if v:
                    os.environ[k] = v  # read when the handle is created
                else:
                    os.environ.pop(k, None)
            probs = _random_batch(g)
            rows_per_wave = int(g.choice([0, 0, 1, 4, 8, 12, 16]))  # work-item size of the level kernel
            res, sess = gpu_run(probs, algo=algo, max_total_time_ns=width, rows_per_wave=rows_per_wave)
            with sess:
                assert_results_match(probs, res, threads=0)
                small = [q for q, p in enumerate(probs) if p["time_ns"].shape[0] <= 66]
                if small:
                    q = small[int(g.integers(0, len(small)))]
                    assert_tables_match(probs[q], sess, q, threads=0)
    finally:
        for k, v in saved.items():
            if v is None:
                os.environ.pop(k, None)
            else:
                os.environ[k] = v
