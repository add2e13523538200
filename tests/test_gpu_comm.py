"""GPU parity of the communication term of the stage time (Sec. III-C: a stage that has a
follower also sends its outputs to it) against the CPU oracle: tables, values, plans, status
words, and the outer driver with the term.  Integers: bit-exact."""
import numpy as np
import pytest
import torch

import oracle
from paper_2103_16063_amd import binding as B
from paper_2103_16063_amd import synth
from tests import defcheck
from tests.gpu_util import INF, assert_results_match, assert_tables_match, gpu_run

pytestmark = pytest.mark.gpu

ALGOS = [B.ALGO_MERGE, B.ALGO_SCAN]
WIDTHS = [B.NARROW_MAX_TOTAL_TIME, 1 << 50]
SHAPES = [(1, 1, 1), (1, 7, 3), (9, 1, 4), (5, 2, 5), (16, 4, 4), (33, 5, 5), (63, 8, 8), (64, 9, 6),
          (65, 12, 7), (100, 17, 9), (129, 24, 6), (130, 33, 5), (200, 40, 4), (70, 63, 10), (96, 64, 12)]


@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("width", WIDTHS)
def test_shape_sweep_with_comm(algo, width):
    for n, (N, D, S) in enumerate(SHAPES):
        for tight, w in ((1.3, 1000), (2.0, 37), (40.0, 250)):
            pr = synth.random_small(1900 + n, N, D, S, tight=tight, tmax=5000)
            pr = synth.with_cut_bytes(pr, 50 + n, w, lo=0, hi=4000 * w // 1000, zero_frac=0.1)
            if width > B.NARROW_MAX_TOTAL_TIME:
                pr["time_ns"] = pr["time_ns"] * (1 << 24)  # totals beyond 32 bits
                pr["cut_bytes"] = pr["cut_bytes"] * (1 << 24)
            res, sess = gpu_run([pr], algo=algo, max_total_time_ns=width)
            with sess:
                assert_results_match([pr], res)
                assert_tables_match(pr, sess, 0, args=(N <= 100))


@pytest.mark.parametrize("fused", ["0", "2"])
def test_mixed_batch_with_and_without_comm(monkeypatch, fused):
    """One batch holding searches with the term, without it (zero bytes on every cut) and with
    different bandwidths, through the one-launch kernel and through the launch per level."""
    monkeypatch.setenv("RANNC_DP_FUSED_SMALL", fused)
    probs = []
    for seed in range(40):
        g = np.random.default_rng(88_000 + seed)
        N, D = int(g.integers(1, 129)), int(g.integers(1, 65))
        pr = synth.random_small(seed, N, D, int(g.integers(1, 20)), tight=float(g.choice([1.2, 2.0, 9.0])),
                                tmax=int(g.choice([7, 3000])))
        if seed % 3:
            w = int(g.choice([1, 90, 1000, 100_000]))
            pr = synth.with_cut_bytes(pr, seed, w, lo=0, hi=max(1, 3 * w), zero_frac=0.2)
        probs.append(pr)
    res, sess = gpu_run(probs)
    with sess:
        assert_results_match(probs, res)
        for q in (1, 2, 7, 20):
            assert_tables_match(probs[q], sess, q, args=False)
    changed = 0
    for pr in probs:
        if "cut_bytes" in pr:
            bare = {k: v for k, v in pr.items() if k not in ("cut_bytes", "bandwidth_bytes_per_us")}
            changed += oracle.solve(pr)["opt"] != oracle.solve(bare)["opt"]
    assert changed >= 5, changed


@pytest.mark.parametrize("k", [2, 3])
def test_named_configs_with_comm(k):
    """The BERT-like and ResNet-like chains with boundary values of 1-64 MiB per microbatch at
    100 GB/s (bytes per microsecond = 100 000): the term is of the order of a block's time."""
    pr = synth.with_cut_bytes(synth.named_config(k), 17, 100_000, lo=1 << 20, hi=64 << 20)
    res, sess = gpu_run([pr])
    with sess:
        assert_results_match([pr], res)
        assert_tables_match(pr, sess, 0)
        defcheck.check_plan(pr["time_ns"], pr["param_bytes"], pr["act_bytes"], pr["n_devices"],
                            pr["max_stages"], pr["mem_capacity"], int(res["opt"][0]), int(res["n_stages"][0]),
                            res["stage_end"][0], res["replicas"][0],
                            (pr["cut_bytes"], pr["bandwidth_bytes_per_us"]))


def test_config4_with_comm_full_size():
    pr = synth.with_cut_bytes(synth.named_config(4), 4, 100_000, lo=1 << 20, hi=32 << 20)
    res, sess = gpu_run([pr])
    with sess:
        assert_results_match([pr], res)
        assert_tables_match(pr, sess, 0, args=False)
    bare = synth.named_config(4)
    assert int(res["opt"][0]) > oracle.solve(bare, n_threads=0)["opt"]


def test_comm_status_words_and_rejections():
    base = synth.random_small(1, 12, 4, 3, tight=3.0)
    good = synth.with_cut_bytes(base, 1, 1000, lo=0, hi=500)
    neg = dict(good); neg["cut_bytes"] = good["cut_bytes"].copy(); neg["cut_bytes"][11] = -1  # last block too
    ovf = dict(good); ovf["cut_bytes"] = good["cut_bytes"].copy(); ovf["cut_bytes"][3] = (((1 << 62) - 1) // 1000) + 1
    edge = dict(good); edge["cut_bytes"] = good["cut_bytes"].copy(); edge["cut_bytes"][3] = ((1 << 62) - 1) // 1000
    edge["bandwidth_bytes_per_us"] = 1 << 50
    big = dict(good); big["cut_bytes"] = good["cut_bytes"].copy(); big["cut_bytes"][2] = 5_000_000_000  # 5e9 ns at 1000 B/us
    lastbig = dict(good); lastbig["cut_bytes"] = good["cut_bytes"].copy(); lastbig["cut_bytes"][11] = 5_000_000_000
    res, sess = gpu_run([good, neg, ovf, big, lastbig, edge])
    with sess:
        assert list(res["status"]) == [B.PROBLEM_OK, B.PROBLEM_NEGATIVE_INPUT, B.PROBLEM_SUM_OVERFLOW,
                                       B.PROBLEM_TIME_TOO_LARGE, B.PROBLEM_OK, B.PROBLEM_OK]
        for q in (1, 2, 3):
            assert res["opt"][q] == INF and res["n_stages"][q] == 0
        for q in (0, 4, 5):
            assert_results_match([[good, 0, 0, 0, lastbig, edge][q]], {k: v[[q]] for k, v in res.items()})
        # bandwidth without bytes, and a bandwidth below 1
        hb = B.HostBatch(*[sess.batch_np[k] for k in ("n_blocks", "n_devices", "max_stages", "n_microbatches",
                                                       "mem_capacity", "block_offset")], *sess.d_in,
                         sess.batch_np["bandwidth_bytes_per_us"], None)
        assert B.rannc_dp_solve(sess.h, hb, sess.stream(), sess.d_opt, sess.d_ns) == B.INVALID_ARG
        bw0 = sess.batch_np["bandwidth_bytes_per_us"].copy(); bw0[2] = 0
        hb = B.HostBatch(*[sess.batch_np[k] for k in ("n_blocks", "n_devices", "max_stages", "n_microbatches",
                                                       "mem_capacity", "block_offset")], *sess.d_in, bw0, sess.d_cut)
        assert B.rannc_dp_solve(sess.h, hb, sess.stream(), sess.d_opt, sess.d_ns) == B.INVALID_ARG
        torch.cuda.synchronize()
    # the same long send time is fine on a 64-bit handle
    res, sess = gpu_run([big], max_total_time_ns=1 << 60)
    with sess:
        assert_results_match([big], res)


FS_CASES = []
for seed in range(24):
    g = np.random.default_rng(61_000 + seed)
    FS_CASES.append((seed, int(g.integers(2, 40)), int(g.choice([1, 2, 4, 8])), int(g.integers(1, 5)),
                     int(g.choice([4, 8, 16, 64])), float(g.choice([0.6, 1.0, 2.0, 20.0])),
                     int(g.choice([50, 1000, 20_000]))))


@pytest.mark.parametrize("seed,N,n_nodes,d_node,BS,tight,w", FS_CASES)
def test_form_stage_with_comm(seed, N, n_nodes, d_node, BS, tight, w):
    c = synth.form_stage_case(seed, N, n_nodes, d_node, BS, tight=tight, tmax=60)
    os_ = np.random.default_rng(seed).integers(0, max(1, 40 * w // 1000), N, endpoint=True)
    want = oracle.form_stage(c["time_per_sample_ns"], c["act_bytes_per_sample"], c["param_bytes"],
                             n_nodes, d_node, BS, c["mem_capacity"], n_threads=0,
                             cut_bytes_per_sample=os_, bandwidth_bytes_per_us=w)
    fs = B.FormStageSession(N, n_nodes, d_node, BS)
    try:
        rc, out, se, rp = fs.run(c["time_per_sample_ns"], c["act_bytes_per_sample"], c["param_bytes"],
                                 c["mem_capacity"], os_, w)
    finally:
        fs.close()
    assert rc == B.OK
    if want is None:
        assert out.feasible == 0 and (se == -1).all()
        return
    have = {"n": out.n, "devices": out.devices, "replica_factor": out.replica_factor,
            "n_stages": out.n_stages, "n_microbatches": out.n_microbatches,
            "stage_time_ns": out.stage_time_ns, "est_iter_ns": out.est_iter_ns}
    for k, v in have.items():
        assert v == want[k], (k, v, want[k])
    S = want["n_stages"]
    assert np.array_equal(se[:S], want["stage_end"]) and np.array_equal(rp[:S], want["replicas"])
    assert (se[S:] == -1).all() and (rp[S:] == -1).all()
