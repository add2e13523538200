"""Regression pins: the oracle still gives the stored answers on the benchmark configurations
(written by tests/golden/make_golden.py, which calls only the oracle)."""
import json
import os

import pytest

import oracle
from paper_2103_16063_amd import synth

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "oracle_configs.json")))


@pytest.mark.parametrize("k", [1, 2, 3])
def test_small_configs(k):
    pr = synth.named_config(k)
    g = GOLD["configs"][str(k)]
    r = oracle.solve(pr, n_threads=0, keep_tables=True)
    N, D = g["N"], g["D"]
    assert (r["opt"], r["n_stages"], r["est_iter_ns"]) == (g["opt"], g["n_stages"], g["est_iter_ns"])
    assert [int(x) for x in r["stage_end"]] == g["stage_end"]
    assert [int(x) for x in r["replicas"]] == g["replicas"]
    assert [int(x) for x in r["V"][1:, N, D]] == g["V_full_chain_all_devices"]


def test_config5_sample():
    sweep = synth.batched_sweep(Q=4)
    for q in range(4):
        g = GOLD["config5_sample"][str(q)]
        r = oracle.solve(sweep[q], n_threads=0)
        assert (r["opt"], r["n_stages"]) == (g["opt"], g["n_stages"])
        assert [int(x) for x in r["stage_end"]] == g["stage_end"]
