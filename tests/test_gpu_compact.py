"""GPU parity of the compaction step of the block-level phase (Sec. III-B) against the CPU oracle,
and the hand-over of its result, still on the device, to the stage-level search."""
import numpy as np
import pytest
import torch

import oracle
from paper_2103_16063_amd import binding as B
from paper_2103_16063_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def gpu_compact(t, p, a, k, M, walks=0):
    G = len(t)
    d_in = [torch.from_numpy(np.ascontiguousarray(x, dtype=np.int64)).to(DEV) for x in (t, p, a)]
    nbytes = B.rannc_dp_compact_workspace_bytes(G)
    assert nbytes > 0
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    d_n = torch.full((1,), -5, dtype=torch.int32, device=DEV)
    d_st = torch.full((1,), -5, dtype=torch.int32, device=DEV)
    d_end = torch.full((G,), -5, dtype=torch.int32, device=DEV)
    d_out = [torch.full((G,), -5, dtype=torch.int64, device=DEV) for _ in range(3)]
    rc = B.rannc_dp_compact(torch.cuda.current_stream().cuda_stream, G, k, walks, M, *d_in, ws, nbytes, d_n,
                            d_end, *d_out, d_st)
    torch.cuda.synchronize()
    return rc, int(d_n.item()), int(d_st.item()), d_end, d_out


CASES = []
for seed in range(60):
    g = np.random.default_rng(seed)
    G = int(g.integers(1, 200))
    CASES.append((seed, G, int(g.integers(1, G + 3)), int(g.choice([0, 60, 150, 400, 10**9]))))
CASES += [(100, 1500, 96, 3000), (101, 1600, 32, 10**9), (102, 1601, 700, 2500), (103, 5000, 128, 4000),
          (104, 3000, 1, 10**9), (105, 2048, 5, 10**9), (106, 2049, 5, 600), (107, 4100, 9, 10**9),
          (108, 9000, 40, 20000)]  # around and beyond the sizes whose state fits LDS and whose listing is a rank sort


@pytest.mark.parametrize("seed,G,k,M", CASES)
def test_compact_matches_the_oracle(seed, G, k, M):
    g = np.random.default_rng(10_000 + seed)
    t = g.integers(0, 20, G) if seed % 2 else g.integers(0, 10**6, G)   # many equal times / few
    p, a = g.integers(0, 50, G), g.integers(0, 50, G)
    for walks in (0, 1, 3):   # until k groups or a walk without merges; one walk; at most three
        rc, n, st, d_end, d_out = gpu_compact(t, p, a, k, M, walks)
        assert rc == B.OK and st == B.PROBLEM_OK
        end, tt, pp, aa = oracle.compact(t, p, a, k, M, max_passes=walks)
        assert n == len(end), (walks, n, len(end))
        assert np.array_equal(d_end.cpu().numpy()[:n], end)
        for have, want in zip(d_out, (tt, pp, aa)):
            assert np.array_equal(have.cpu().numpy()[:n], want)
        assert (d_end.cpu().numpy()[n:] == -5).all()     # nothing written behind the result
        if walks == 0 and M == 10**9:
            assert n == min(k, G)                        # memory never refuses: k blocks are reached


def test_compact_status_and_rejections():
    t, p, a = np.array([3, 1, 2]), np.array([1, 1, 1]), np.array([1, 1, 1])
    neg = t.copy(); neg[1] = -1
    rc, n, st, *_ = gpu_compact(neg, p, a, 2, 100)
    assert rc == B.OK and st == B.PROBLEM_NEGATIVE_INPUT and n == 0
    big = np.array([1 << 61, 1 << 61, 5])
    rc, n, st, *_ = gpu_compact(t, big, a, 2, 100)
    assert rc == B.OK and st == B.PROBLEM_SUM_OVERFLOW and n == 0
    assert B.rannc_dp_compact_workspace_bytes(0) == 0 and B.rannc_dp_compact_workspace_bytes(70000) == 0
    d = torch.zeros(3, dtype=torch.int64, device=DEV)
    di = torch.zeros(3, dtype=torch.int32, device=DEV)
    ws = torch.empty(4096, dtype=torch.uint8, device=DEV)
    s = torch.cuda.current_stream().cuda_stream
    assert B.rannc_dp_compact(s, 3, 0, 0, 5, d, d, d, ws, 4096, di, di, d, d, d, di) == B.INVALID_ARG
    assert B.rannc_dp_compact(s, 3, 2, 0, -1, d, d, d, ws, 4096, di, di, d, d, d, di) == B.INVALID_ARG
    assert B.rannc_dp_compact(s, 3, 2, -1, 5, d, d, d, ws, 4096, di, di, d, d, d, di) == B.INVALID_ARG
    assert B.rannc_dp_compact(s, 3, 2, 0, 5, d, d, d, ws, 8, di, di, d, d, d, di) == B.WORKSPACE_TOO_SMALL
    assert B.rannc_dp_compact(s, 3, 2, 0, 5, d, None, d, ws, 4096, di, di, d, d, d, di) == B.INVALID_ARG
    torch.cuda.synchronize()


def test_compaction_feeds_the_search_on_the_device():
    """400 fine-grained groups -> compaction to 96 blocks (a single walk would end at 158; repeated
    walks reach 96) -> stage-level search, the block arrays never leaving the device; the same two
    steps on the oracle give the same plan."""
    fine = synth.enlarged_transformer_chain(seed=21, N=400, D=16, S=8, MB=32, M=48 << 30)
    t, p, a = fine["time_ns"], fine["param_bytes"], fine["act_bytes"]
    k, M = 96, fine["mem_capacity"]
    rc, n, st, d_end, d_out = gpu_compact(t, p, a, k, M)
    assert rc == B.OK and st == B.PROBLEM_OK
    end, tt, pp, aa = oracle.compact(t, p, a, k, M)
    assert n == len(end) == k and np.array_equal(d_end.cpu().numpy()[:n], end)
    assert len(oracle.compact(t, p, a, k, M, max_passes=1)[0]) == 158
    # search over the n blocks, inputs = the compaction's device arrays
    lim = B.make_limits(1, n, 16, 8)
    hb = B.HostBatch([n], [16], [8], [32], [M], [0, n], *[x[:n] for x in d_out])
    nbytes = B.rannc_dp_workspace_bytes_for(lim, hb)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    rc, h = B.rannc_dp_create(lim, ws, nbytes)
    assert rc == B.OK
    try:
        d_opt = torch.empty(1, dtype=torch.int64, device=DEV)
        d_ns = torch.empty(1, dtype=torch.int32, device=DEV)
        d_se = torch.empty((1, 8), dtype=torch.int32, device=DEV)
        d_rp = torch.empty((1, 8), dtype=torch.int32, device=DEV)
        s = torch.cuda.current_stream().cuda_stream
        assert B.rannc_dp_solve(h, hb, s, d_opt, d_ns) == B.OK
        assert B.rannc_dp_traceback(h, s, 8, d_se, d_rp) == B.OK
        torch.cuda.synchronize()
    finally:
        B.rannc_dp_destroy(h)
    blocks = {"name": "compacted", "time_ns": tt, "param_bytes": pp, "act_bytes": aa, "n_devices": 16,
              "max_stages": 8, "n_microbatches": 32, "mem_capacity": M}
    o = oracle.solve(blocks, n_threads=0)
    assert int(d_opt.item()) == o["opt"] and int(d_ns.item()) == o["n_stages"] and o["n_stages"] >= 1
    assert np.array_equal(d_se.cpu().numpy()[0], o["stage_end"]) and np.array_equal(d_rp.cpu().numpy()[0], o["replicas"])
