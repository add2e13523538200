"""Writes tests/golden/oracle_configs.json: the oracle's answers for the benchmark's
configurations.  Calls only the input generators and oracle/ (never the HIP path).
The paper prints no worked numeric example of the search, so there is no paper-side
fixture; these values are regression pins of the oracle, which is itself pinned by
tests/test_oracle_pins.py.

    python tests/golden/make_golden.py
"""
import hashlib
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2103_16063_amd import synth  # noqa: E402

C5_SAMPLE = [0, 1, 2, 3, 17, 255, 1024, 2047]


def record(pr, threads=0):
    r = oracle.solve(pr, n_threads=threads, keep_tables=True)
    N, D = pr["time_ns"].shape[0], pr["n_devices"]
    return {
        "name": pr["name"],
        "N": N, "D": D, "S": pr["max_stages"], "MB": pr["n_microbatches"],
        "M": pr["mem_capacity"],
        "opt": r["opt"], "n_stages": r["n_stages"], "est_iter_ns": r["est_iter_ns"],
        "stage_end": [int(x) for x in r["stage_end"]],
        "replicas": [int(x) for x in r["replicas"]],
        "V_full_chain_all_devices": [int(x) for x in r["V"][1:, N, D]],
        "sha256_V": hashlib.sha256(r["V"].tobytes()).hexdigest(),
        "sha256_arg_i": hashlib.sha256(r["arg_i"].tobytes()).hexdigest(),
        "sha256_arg_d": hashlib.sha256(r["arg_d"].tobytes()).hexdigest(),
    }


def main():
    out = {"configs": {}, "config5_sample": {}}
    for k in (1, 2, 3, 4):
        out["configs"][str(k)] = record(synth.named_config(k))
        print("config", k, out["configs"][str(k)]["opt"], out["configs"][str(k)]["n_stages"])
    sweep = synth.batched_sweep()
    for q in C5_SAMPLE:
        out["config5_sample"][str(q)] = record(sweep[q])
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_configs.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1)
    print("wrote", path)


if __name__ == "__main__":
    main()
