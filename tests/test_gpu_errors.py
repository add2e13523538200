"""Error and status paths of the C ABI on a real device (every kernel still exits normally)."""
import numpy as np
import pytest
import torch

from paper_2103_16063_amd import binding as B
from paper_2103_16063_amd import synth
from tests.gpu_util import INF, assert_results_match, gpu_run

pytestmark = pytest.mark.gpu


def test_per_problem_status_words():
    good = synth.random_small(1, 12, 4, 3, tight=3.0)
    neg = synth.random_small(2, 12, 4, 3, tight=3.0)
    neg["act_bytes"] = neg["act_bytes"].copy()
    neg["act_bytes"][5] = -7
    ovf = synth.random_small(3, 12, 4, 3, tight=3.0)
    ovf["param_bytes"] = np.full(12, 1 << 60, dtype=np.int64)
    ovf["mem_capacity"] = (1 << 62)
    big = synth.random_small(4, 12, 4, 3, tight=3.0)
    big["time_ns"] = big["time_ns"] * (1 << 30)
    res, sess = gpu_run([good, neg, ovf, big, good])
    with sess:
        assert list(res["status"]) == [B.PROBLEM_OK, B.PROBLEM_NEGATIVE_INPUT, B.PROBLEM_SUM_OVERFLOW,
                                       B.PROBLEM_TIME_TOO_LARGE, B.PROBLEM_OK]
        for q in (1, 2, 3):
            assert res["opt"][q] == INF and res["n_stages"][q] == 0
            assert (res["stage_end"][q] == -1).all() and (res["replicas"][q] == -1).all()
        assert_results_match([good], {k: v[[0]] for k, v in res.items()})
        assert_results_match([good], {k: v[[4]] for k, v in res.items()})
    # the same large-time problem is fine on a 64-bit handle
    res, sess = gpu_run([big], max_total_time_ns=1 << 60)
    with sess:
        assert_results_match([big], res)


def test_host_side_rejections():
    pr = synth.random_small(1, 20, 4, 3)
    b = synth.concat_batch([pr])
    sess = B.Session(b)
    with sess:
        # traceback / export before any solve
        assert B.rannc_dp_traceback(sess.h, sess.stream(), 4, sess.d_se, sess.d_rp) == B.BAD_STATE
        assert B.rannc_dp_read_table(sess.h, B.TABLE_V, 0, sess.d_se, 8, sess.stream()) == B.BAD_STATE
        sess.solve()
        assert B.rannc_dp_traceback(sess.h, sess.stream(), 2, sess.d_se, sess.d_rp) == B.INVALID_ARG
        assert B.rannc_dp_read_table(sess.h, B.TABLE_V, 0, sess.d_se, 8, sess.stream()) == B.INVALID_ARG
        assert B.rannc_dp_read_table(sess.h, B.TABLE_V, 3, sess.d_se, 8, sess.stream()) == B.INVALID_ARG
        assert B.rannc_dp_read_table(sess.h, 9, 0, sess.d_se, 8, sess.stream()) == B.INVALID_ARG
        # a batch beyond the handle's limits
        pr2 = synth.random_small(1, 21, 4, 3)
        hb2 = B.Session.__new__(B.Session)
        b2 = synth.concat_batch([pr2])
        d_in = [torch.from_numpy(b2[k]).to("cuda:0") for k in ("time_ns", "param_bytes", "act_bytes")]
        hb = B.HostBatch(b2["n_blocks"], b2["n_devices"], b2["max_stages"], b2["n_microbatches"],
                         b2["mem_capacity"], b2["block_offset"], *d_in)
        assert B.rannc_dp_solve(sess.h, hb, sess.stream(), sess.d_opt, sess.d_ns) == B.LIMIT_EXCEEDED
        bad = dict(b)
        bad["n_microbatches"] = np.array([0], dtype=np.int32)
        hb = B.HostBatch(bad["n_blocks"], bad["n_devices"], bad["max_stages"], bad["n_microbatches"],
                         bad["mem_capacity"], bad["block_offset"], *sess.d_in)
        assert B.rannc_dp_solve(sess.h, hb, sess.stream(), sess.d_opt, sess.d_ns) == B.INVALID_ARG
        assert B.rannc_dp_solve(sess.h, sess.hb, sess.stream(), None, sess.d_ns) == B.INVALID_ARG
        torch.cuda.synchronize()


def test_workspace_too_small_is_reported():
    pr = synth.random_small(1, 100, 16, 4)
    b = synth.concat_batch([pr])
    lim = B.make_limits(1, 100, 16, 4)
    ws = torch.empty(1 << 16, dtype=torch.uint8, device="cuda:0")
    rc, h = B.rannc_dp_create(lim, ws, ws.numel())
    assert rc == B.OK
    d_in = [torch.from_numpy(b[k]).to("cuda:0") for k in ("time_ns", "param_bytes", "act_bytes")]
    hb = B.HostBatch(b["n_blocks"], b["n_devices"], b["max_stages"], b["n_microbatches"],
                     b["mem_capacity"], b["block_offset"], *d_in)
    d_opt = torch.empty(1, dtype=torch.int64, device="cuda:0")
    d_ns = torch.empty(1, dtype=torch.int32, device="cuda:0")
    assert B.rannc_dp_solve(h, hb, None, d_opt, d_ns) == B.WORKSPACE_TOO_SMALL
    B.rannc_dp_destroy(h)


def test_worst_case_workspace_and_handle_reuse():
    """One handle sized from its limits serves batches of different shapes one after another."""
    probs_a = [synth.random_small(50 + q, 60, 8, 5, tight=1.5) for q in range(6)]
    probs_b = [synth.random_small(80 + q, 17, 3, 2, tight=1.5) for q in range(3)]
    sa = B.Session(synth.concat_batch(probs_a), exact_workspace=False)
    with sa:
        res_a = sa.run()
        assert_results_match(probs_a, res_a)
        bb = synth.concat_batch(probs_b)
        d_in = [torch.from_numpy(bb[k]).to("cuda:0") for k in ("time_ns", "param_bytes", "act_bytes")]
        hb = B.HostBatch(bb["n_blocks"], bb["n_devices"], bb["max_stages"], bb["n_microbatches"],
                         bb["mem_capacity"], bb["block_offset"], *d_in)
        assert B.rannc_dp_solve(sa.h, hb, sa.stream(), sa.d_opt, sa.d_ns, sa.d_est, sa.d_status) == B.OK
        assert B.rannc_dp_traceback(sa.h, sa.stream(), sa.plan_stride, sa.d_se, sa.d_rp) == B.OK
        torch.cuda.synchronize()
        res_b = {"opt": sa.d_opt.cpu().numpy()[:3], "n_stages": sa.d_ns.cpu().numpy()[:3],
                 "est_iter_ns": sa.d_est.cpu().numpy()[:3], "status": sa.d_status.cpu().numpy()[:3],
                 "stage_end": sa.d_se.cpu().numpy()[:3], "replicas": sa.d_rp.cpu().numpy()[:3]}
        assert_results_match(probs_b, res_b)


def test_timing_events():
    pr = synth.named_config(2)
    sess = B.Session(synth.concat_batch([pr]))
    with sess:
        rc, _, _ = B.rannc_dp_get_timing(sess.h)
        assert rc == B.BAD_STATE
        B.rannc_dp_set_timing(sess.h, True)
        sess.run()
        rc, ms, n = B.rannc_dp_get_timing(sess.h)
        assert rc == B.OK and n >= 1 and all(m >= 0 for m in ms) and ms[1] > 0


def test_totals_at_the_edge_of_32_bit_tables():
    """A total time of exactly 2^32 - 2 ns still fits 32-bit tables (2^32 - 1 is the "no plan" mark);
    one more nanosecond is reported as too large.  Same with a send time on top."""
    edge = synth.random_small(9, 6, 4, 3, tight=4.0)
    edge["time_ns"] = np.array([B.NARROW_MAX_TOTAL_TIME - 5, 1, 1, 1, 1, 1], dtype=np.int64)
    over = dict(edge)
    over["time_ns"] = edge["time_ns"].copy(); over["time_ns"][3] = 2
    comm_edge = synth.with_cut_bytes(dict(edge), 1, 1000, lo=0, hi=0)
    comm_edge["time_ns"] = edge["time_ns"].copy(); comm_edge["time_ns"][0] -= 7
    comm_edge["cut_bytes"] = np.array([0, 7, 3, 0, 1, 10**9], dtype=np.int64)   # longest send: 7 ns; last cut unused
    comm_over = dict(comm_edge); comm_over["cut_bytes"] = np.array([0, 8, 3, 0, 1, 0], dtype=np.int64)
    res, sess = gpu_run([edge, over, comm_edge, comm_over])
    with sess:
        assert list(res["status"]) == [B.PROBLEM_OK, B.PROBLEM_TIME_TOO_LARGE, B.PROBLEM_OK, B.PROBLEM_TIME_TOO_LARGE]
        assert_results_match([edge], {k: v[[0]] for k, v in res.items()})
        assert_results_match([comm_edge], {k: v[[2]] for k, v in res.items()})
        assert int(res["opt"][0]) != INF
