"""Helpers for the GPU parity tests: run problems through the C ABI, run the oracle on the
same seeded inputs, compare element by element (integers: bit-exact)."""
import numpy as np

import oracle
from paper_2103_16063_amd import binding as B
from paper_2103_16063_amd import synth

INF = B.INT64_MAX


def gpu_run(problems, **kw):
    """(results, session) for a list of problem dicts solved as one batch."""
    sess = B.Session(synth.concat_batch(problems), **kw)
    return sess.run(), sess


def oracle_solve_many(problems, workers=None):
    """oracle.solve of every problem, one search per host thread (the C calls release the GIL)."""
    import os
    from concurrent.futures import ThreadPoolExecutor
    workers = workers or min(16, os.cpu_count() or 1)
    with ThreadPoolExecutor(max_workers=workers) as ex:
        return list(ex.map(lambda pr: oracle.solve(pr, n_threads=1), problems))


def assert_results_match(problems, res, threads=0, oracle_results=None):
    for q, pr in enumerate(problems):
        o = oracle_results[q] if oracle_results is not None else oracle.solve(pr, n_threads=threads)
        S_eff = o["n_levels"]
        assert int(res["status"][q]) == 0, (q, pr["name"])
        assert int(res["opt"][q]) == o["opt"], (q, pr["name"], int(res["opt"][q]), o["opt"])
        assert int(res["n_stages"][q]) == o["n_stages"], (q, pr["name"])
        assert int(res["est_iter_ns"][q]) == o["est_iter_ns"], (q, pr["name"])
        se, rp = res["stage_end"][q], res["replicas"][q]
        k = min(len(se), len(o["stage_end"]))
        assert S_eff <= len(se)
        assert np.array_equal(se[:k], o["stage_end"][:k]), (q, pr["name"], se, o["stage_end"])
        assert np.array_equal(rp[:k], o["replicas"][:k]), (q, pr["name"], rp, o["replicas"])
        assert (se[k:] == -1).all() and (rp[k:] == -1).all()


def assert_tables_match(pr, sess, q, threads=0, args=True):
    o = oracle.solve(pr, n_threads=threads, keep_tables=True)
    fit = sess.table(B.TABLE_FIT, q)
    assert np.array_equal(fit, o["fit"]), pr["name"]
    cost = sess.table(B.TABLE_COST, q)
    assert np.array_equal(cost, np.where(o["fit"] != 0, o["cost"], INF)), pr["name"]
    V = sess.table(B.TABLE_V, q)
    assert V.shape == o["V"].shape
    if not np.array_equal(V, o["V"]):
        bad = np.argwhere(V != o["V"])
        raise AssertionError(f"{pr['name']}: V differs at {len(bad)} cells, first (s,j,d)={bad[0]} "
                             f"gpu={V[tuple(bad[0])]} oracle={o['V'][tuple(bad[0])]}")
    if "time_bwd_ns" in pr:  # split objective: second stage-time table and the two carried maxima
        cb = sess.table(B.TABLE_COST_BWD, q)
        assert np.array_equal(cb, np.where(o["fit"] != 0, o["cost_bwd"], INF)), pr["name"]
        assert np.array_equal(sess.table(B.TABLE_MAX_FWD, q), o["TF"]), pr["name"]
        assert np.array_equal(sess.table(B.TABLE_MAX_BWD, q), o["TB"]), pr["name"]
    if args:
        ai = sess.table(B.TABLE_ARG_I, q)
        ad = sess.table(B.TABLE_ARG_D, q)
        assert np.array_equal(ai, o["arg_i"]), pr["name"]
        assert np.array_equal(ad, o["arg_d"]), pr["name"]
    return o
