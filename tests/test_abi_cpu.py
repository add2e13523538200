"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
public header declares, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2103_16063_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "rannc_dp.h")).read()
    return sorted(set(re.findall(r"RANNC_DP_API[^;(]*?\b(rannc_dp_\w+)\s*\(", text)))


def test_library_is_built():
    assert os.path.exists(B.LIB_PATH), "run python -m paper_2103_16063_amd.build"


def test_exports_every_declared_symbol():
    names = _declared()
    assert len(names) >= 10 and set(names) == set(B.EXPORTS)
    L = C.CDLL(B.LIB_PATH, mode=os.RTLD_NOW)  # resolve everything now: an undefined symbol fails here
    for n in names:
        assert hasattr(L, n), n


def test_strerror_is_total():
    for code in range(-9, 2):
        assert isinstance(B.strerror(code), str) and B.strerror(code)
    assert B.strerror(0) == "ok"


def test_workspace_query_validates():
    assert B.rannc_dp_workspace_bytes(B.make_limits(0, 16, 4, 4)) == 0
    assert B.rannc_dp_workspace_bytes(B.make_limits(1, 0, 4, 4)) == 0
    assert B.rannc_dp_workspace_bytes(B.make_limits(1, 16, 65, 4)) == 0
    assert B.rannc_dp_workspace_bytes(B.make_limits(1, 16, 4, 0)) == 0
    assert B.rannc_dp_workspace_bytes(B.make_limits(1, 16, 4, 4, max_total_time_ns=-1)) == 0
    assert B.rannc_dp_workspace_bytes(B.make_limits(1, 16, 4, 4, algo=7)) == 0
    assert B.rannc_dp_workspace_bytes(B.make_limits(1, 16, 4, 4, algo=B.ALGO_RECOMPUTE)) > 0
    assert B.rannc_dp_workspace_bytes(B.make_limits(1, 16, 4, 4, rows_per_wave=17)) == 0     # tuning out of range
    assert B.rannc_dp_workspace_bytes(B.make_limits(1, 16, 4, 4, one_launch_small=3)) == 0
    assert B.rannc_dp_workspace_bytes(B.make_limits(1, 16, 4, 4, single_stream=2)) == 0
    assert B.rannc_dp_workspace_bytes(B.make_limits(1, 16, 4, 4, rows_per_wave=8, one_launch_small=2, single_stream=1)) > 0
    small = B.rannc_dp_workspace_bytes(B.make_limits(1, 16, 4, 4))
    big = B.rannc_dp_workspace_bytes(B.make_limits(1, 1024, 64, 32))
    wide = B.rannc_dp_workspace_bytes(B.make_limits(1, 1024, 64, 32, max_total_time_ns=1 << 40))
    assert 0 < small < big < wide
    # 32-bit tables of config 4: 64 * 64 * sum over rows of the padded row length * 4 bytes
    assert big > 64 * 1024 * 1025 // 2 * 4
    assert B.rannc_dp_workspace_bytes(B.make_limits(8, 1024, 64, 32)) > 7 * big


def _host_batch(N=4, D=2, S=2, MB=1, M=100, off=None):
    z = np.zeros(N, dtype=np.int64)
    off = np.array([0, N], dtype=np.int64) if off is None else off
    # fake non-null device addresses: never dereferenced by the size query
    hb = B.HostBatch([N], [D], [S], [MB], [M], off, z, z, z)
    return hb


def test_exact_workspace_query():
    lim = B.make_limits(1, 64, 8, 8)
    assert 0 < B.rannc_dp_workspace_bytes_for(lim, _host_batch()) <= B.rannc_dp_workspace_bytes(lim)
    assert B.rannc_dp_workspace_bytes_for(lim, _host_batch(N=65)) == 0  # exceeds limits
    assert B.rannc_dp_workspace_bytes_for(lim, _host_batch(D=9)) == 0
    assert B.rannc_dp_workspace_bytes_for(lim, _host_batch(M=-1)) == 0
    assert B.rannc_dp_workspace_bytes_for(lim, _host_batch(off=np.array([0, 3], dtype=np.int64))) == 0


def test_create_rejects_bad_arguments_before_any_device_work():
    lim = B.make_limits(1, 16, 4, 4)
    rc, h = B.rannc_dp_create(lim, None, 1 << 20)
    assert rc == B.INVALID_ARG and h is None
    rc, h = B.rannc_dp_create(lim, 0x1001, 1 << 20)  # misaligned
    assert rc == B.INVALID_ARG and h is None
    rc, h = B.rannc_dp_create(B.make_limits(1, 16, 400, 4), 0x1000, 1 << 20)
    assert rc == B.INVALID_ARG and h is None
    rc, h = B.rannc_dp_create(lim, 0x1000, 16)
    assert rc == B.WORKSPACE_TOO_SMALL and h is None


def test_null_handle_calls():
    assert B.rannc_dp_solve(None, None, None, None, None) == B.INVALID_ARG
    assert B.rannc_dp_traceback(None, None, 4, None, None) == B.INVALID_ARG
    assert B.rannc_dp_read_table(None, 0, 0, None, 0, None) == B.INVALID_ARG
    assert B.rannc_dp_set_timing(None, True) == B.INVALID_ARG
    B.rannc_dp_destroy(None)


def test_form_stage_host_queries():
    """Number of searches the outer driver issues = the (node count, microbatch count) pairs
    Algorithm 2 can visit: n = 1, 2, 4, ... <= n_nodes, MB = 1, 2, 4, ... <= floor(BS / (n_nodes / n))."""
    z = np.zeros(8, dtype=np.int64)

    def pairs(n_nodes, d_node, BS):
        return B.rannc_dp_form_stage_problems(B.HostFormStageIn(z, z, z, n_nodes, d_node, BS, 1))

    assert pairs(1, 8, 1) == 1
    assert pairs(1, 8, 256) == 9                      # MB = 1 .. 256
    assert pairs(4, 8, 256) == 7 + 8 + 9              # R = 4, 2, 1 -> BS/R = 64, 128, 256
    assert pairs(3, 2, 8) == 2 + 4                    # n = 1 (R = 3, MB <= 2), n = 2 (R = 1, MB = 1, 2, 4, 8)
    assert pairs(4, 8, 2) == 0 + 1 + 2                # BS / R = 0 for n = 1: no microbatch count at all
    assert pairs(16, 8, 64) == 0                      # 8 * 16 devices: more than the kernels hold
    assert pairs(0, 8, 64) == 0 and pairs(2, 0, 64) == 0 and pairs(2, 8, 0) == 0
    small = B.rannc_dp_form_stage_scratch_bytes(B.HostFormStageIn(z, z, z, 1, 8, 1, 1))
    big = B.rannc_dp_form_stage_scratch_bytes(B.HostFormStageIn(z, z, z, 4, 8, 256, 1))
    assert 0 < small < big and small % 256 == 0 and big % 256 == 0
    assert B.rannc_dp_form_stage_scratch_bytes(B.HostFormStageIn(z, z, z, 16, 8, 64, 1)) == 0
    # a communication term needs a bandwidth
    assert B.rannc_dp_form_stage_problems(B.HostFormStageIn(z, z, z, 2, 4, 8, 1, z, 0)) == 0
    assert B.rannc_dp_form_stage_problems(B.HostFormStageIn(z, z, z, 2, 4, 8, 1, z, 5)) == 3 + 4


def test_split_and_compact_host_queries():
    plain = B.rannc_dp_workspace_bytes(B.make_limits(1, 256, 32, 16))
    split = B.rannc_dp_workspace_bytes(B.make_limits(1, 256, 32, 16, flags=B.FLAG_SPLIT_OBJECTIVE))
    assert split > 2 * plain - (1 << 16)              # a second table, two more value tables, the keys
    assert B.rannc_dp_workspace_bytes(B.make_limits(1, 256, 32, 16, flags=4)) == 0
    assert B.rannc_dp_compact_workspace_bytes(1) > 0
    assert B.rannc_dp_compact_workspace_bytes(1600) < B.rannc_dp_compact_workspace_bytes(1601)  # state leaves LDS
    assert B.rannc_dp_compact_workspace_bytes(65535) > 0 and B.rannc_dp_compact_workspace_bytes(65536) == 0
    assert B.rannc_dp_compact(None, 0, 1, 0, 1, None, None, None, None, 0, None, None, None, None, None, None) == B.INVALID_ARG
    assert B.rannc_dp_form_stage(None, B.HostFormStageIn(np.zeros(2), np.zeros(2), np.zeros(2), 1, 1, 1, 1),
                                 None, None, 0, 4)[0] == B.INVALID_ARG
    assert B.rannc_dp_level_values(None, None, 4, None) == B.INVALID_ARG
    assert B.rannc_dp_traceback_at(None, None, None, 4, None, None) == B.INVALID_ARG
