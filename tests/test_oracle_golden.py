"""Regression pins: the oracle still gives the stored answers on the benchmark configurations
(written by tests/golden/make_golden.py, which calls only the oracle)."""
import hashlib
import json
import os

import pytest

import oracle
from paper_2103_16063_amd import synth

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "oracle_configs.json")))


def _sha(a):
    return hashlib.sha256(a.tobytes()).hexdigest()


@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_named_configs(k):
    """Optimum, plan, the column V[s][N][D] and the digests of the whole value and (i, d') tables
    (config 4 included: a few seconds with all host threads)."""
    pr = synth.named_config(k)
    g = GOLD["configs"][str(k)]
    r = oracle.solve(pr, n_threads=0, keep_tables=True)
    assert (_sha(r["V"]), _sha(r["arg_i"]), _sha(r["arg_d"])) == (g["sha256_V"], g["sha256_arg_i"], g["sha256_arg_d"])
    N, D = g["N"], g["D"]
    assert (r["opt"], r["n_stages"], r["est_iter_ns"]) == (g["opt"], g["n_stages"], g["est_iter_ns"])
    assert [int(x) for x in r["stage_end"]] == g["stage_end"]
    assert [int(x) for x in r["replicas"]] == g["replicas"]
    assert [int(x) for x in r["V"][1:, N, D]] == g["V_full_chain_all_devices"]


def test_config5_sample():
    sweep = synth.batched_sweep()
    for key, g in GOLD["config5_sample"].items():
        r = oracle.solve(sweep[int(key)], n_threads=0, keep_tables=True)
        assert (r["opt"], r["n_stages"], r["est_iter_ns"]) == (g["opt"], g["n_stages"], g["est_iter_ns"])
        assert [int(x) for x in r["stage_end"]] == g["stage_end"]
        assert [int(x) for x in r["replicas"]] == g["replicas"]
        assert (_sha(r["V"]), _sha(r["arg_i"]), _sha(r["arg_d"])) == (g["sha256_V"], g["sha256_arg_i"], g["sha256_arg_d"])
