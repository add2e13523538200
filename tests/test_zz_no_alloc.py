"""The compaction entry point that allocates nothing (its workspace is a fixed array inside the
library's device image) against the entry point that takes a caller's workspace: same outputs,
on two calls in a row, the second with a smaller input (the array keeps the first call's contents)."""
import numpy as np
import pytest
import torch

from paper_2103_16063_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run(static, t, p, a, k, M, walks):
    G = len(t)
    d_in = [torch.from_numpy(np.ascontiguousarray(x, dtype=np.int64)).to(DEV) for x in (t, p, a)]
    d_n = torch.full((1,), -5, dtype=torch.int32, device=DEV)
    d_st = torch.full((1,), -5, dtype=torch.int32, device=DEV)
    d_end = torch.full((G,), -5, dtype=torch.int32, device=DEV)
    d_out = [torch.full((G,), -5, dtype=torch.int64, device=DEV) for _ in range(3)]
    s = torch.cuda.current_stream().cuda_stream
    if static:
        rc = B.rannc_dp_compact_static(s, G, k, walks, M, *d_in, d_n, d_end, *d_out, d_st)
    else:
        nbytes = B.rannc_dp_compact_workspace_bytes(G)
        ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
        rc = B.rannc_dp_compact(s, G, k, walks, M, *d_in, ws, nbytes, d_n, d_end, *d_out, d_st)
    torch.cuda.synchronize()
    assert rc == B.OK
    return [x.cpu().numpy() for x in (d_n, d_st, d_end, *d_out)]


def test_static_workspace_entry_point_matches_on_two_calls_in_a_row():
    g = np.random.default_rng(77)
    # first a chain whose state lives in the workspace (beyond the LDS size) and whose listing is
    # the bitonic sort, then a much smaller one whose workspace still holds the first call's data
    for G, k, M, walks in ((6000, 50, 5000, 0), (700, 9, 900, 0), (1601, 3, 10**9, 2), (40, 4, 150, 1)):
        t = g.integers(0, 1000, G)
        p, a = g.integers(0, 50, G), g.integers(0, 50, G)
        want = run(False, t, p, a, k, M, walks)
        have = run(True, t, p, a, k, M, walks)
        assert int(want[1][0]) == B.PROBLEM_OK
        for w, h in zip(want, have):
            assert np.array_equal(w, h), (G, k, M, walks)


def test_static_workspace_entry_point_limits_and_arguments():
    d = torch.zeros(3, dtype=torch.int64, device=DEV)
    di = torch.zeros(3, dtype=torch.int32, device=DEV)
    s = torch.cuda.current_stream().cuda_stream
    big = B.COMPACT_STATIC_MAX_GROUPS + 1
    assert B.rannc_dp_compact_static(s, big, 2, 0, 5, d, d, d, di, di, d, d, d, di) == B.LIMIT_EXCEEDED
    assert B.rannc_dp_compact_static(s, 3, 0, 0, 5, d, d, d, di, di, d, d, d, di) == B.INVALID_ARG
    assert B.rannc_dp_compact_static(s, 3, 2, 0, 5, d, None, d, di, di, d, d, d, di) == B.INVALID_ARG
    # the largest size the array serves
    G = B.COMPACT_STATIC_MAX_GROUPS
    g = np.random.default_rng(3)
    t, p, a = g.integers(0, 10**6, G), g.integers(0, 50, G), g.integers(0, 50, G)
    for w, h in zip(run(False, t, p, a, 64, 3000, 0), run(True, t, p, a, 64, 3000, 0)):
        assert np.array_equal(w, h)
    torch.cuda.synchronize()
