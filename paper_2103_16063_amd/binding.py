"""ctypes binding of the C ABI in include/rannc_dp.h: the same entry points under the same
names, with torch tensors / numpy arrays marshalled to raw pointers.  No step of the search
runs here -- every value comes out of the HIP kernels behind the library.  PyTorch is used
only to own device memory and to provide the stream.

The library must have been built (python -m paper_2103_16063_amd.build); loading fails loudly
otherwise.  There is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librannc_dp.so")

INT64_MAX = (1 << 63) - 1

OK, INVALID_ARG, LIMIT_EXCEEDED, WORKSPACE_TOO_SMALL, OVERFLOW, HIP_ERROR, BAD_STATE, NO_HOST_MEMORY = \
    0, -1, -2, -3, -4, -5, -6, -7
PROBLEM_OK, PROBLEM_NEGATIVE_INPUT, PROBLEM_SUM_OVERFLOW, PROBLEM_TIME_TOO_LARGE = 0, 1, 2, 3
ALGO_AUTO, ALGO_MERGE, ALGO_SCAN, ALGO_RECOMPUTE = 0, 1, 2, 3
TABLE_COST, TABLE_FIT, TABLE_V, TABLE_ARG_I, TABLE_ARG_D = 0, 1, 2, 3, 4
TABLE_COST_BWD, TABLE_MAX_FWD, TABLE_MAX_BWD = 5, 6, 7
FLAG_SPLIT_OBJECTIVE = 1
MAX_DEVICES = 64
NARROW_MAX_TOTAL_TIME = 4294967294
WIDE_RECOMPUTE_MAX_TOTAL_TIME = 1 << 40   # 64-bit handles up to this bound can recompute stage times

EXPORTS = ["rannc_dp_workspace_bytes", "rannc_dp_workspace_bytes_for", "rannc_dp_create",
           "rannc_dp_solve", "rannc_dp_traceback", "rannc_dp_read_table", "rannc_dp_destroy",
           "rannc_dp_strerror", "rannc_dp_set_timing", "rannc_dp_get_timing",
           "rannc_dp_traceback_at", "rannc_dp_level_values", "rannc_dp_form_stage_problems",
           "rannc_dp_form_stage_scratch_bytes", "rannc_dp_form_stage",
           "rannc_dp_compact_workspace_bytes", "rannc_dp_compact", "rannc_dp_compact_static",
           "rannc_dp_solve_info"]


class Limits(C.Structure):
    _fields_ = [("max_problems", C.c_int32), ("max_blocks", C.c_int32),
                ("max_devices", C.c_int32), ("max_stages", C.c_int32),
                ("max_total_time_ns", C.c_int64), ("algo", C.c_int32), ("flags", C.c_int32),
                ("rows_per_wave", C.c_int32), ("one_launch_small", C.c_int32),
                ("single_stream", C.c_int32), ("reserved", C.c_int32)]


class SolveInfo(C.Structure):
    _fields_ = [("n_problems", C.c_int32 * 4), ("level_kernel", C.c_int32 * 4)]


KERNEL_NONE, KERNEL_MERGE_TABLE, KERNEL_MERGE_RECOMPUTE, KERNEL_ONE_LAUNCH, KERNEL_SCAN, KERNEL_SPLIT, \
    KERNEL_SPLIT_SCAN, KERNEL_ONE_LAUNCH_RECOMPUTE = range(8)


class Batch(C.Structure):
    _fields_ = [("n_problems", C.c_int32),
                ("n_blocks", C.c_void_p), ("n_devices", C.c_void_p), ("max_stages", C.c_void_p),
                ("n_microbatches", C.c_void_p), ("mem_capacity", C.c_void_p),
                ("block_offset", C.c_void_p),
                ("time_ns", C.c_void_p), ("param_bytes", C.c_void_p), ("act_bytes", C.c_void_p),
                ("bandwidth_bytes_per_us", C.c_void_p), ("cut_bytes", C.c_void_p),
                ("time_bwd_ns", C.c_void_p)]


class FormStageIn(C.Structure):
    _fields_ = [("n_blocks", C.c_int32), ("n_nodes", C.c_int32), ("devices_per_node", C.c_int32),
                ("reserved", C.c_int32), ("batch_size", C.c_int64), ("mem_capacity", C.c_int64),
                ("time_per_sample_ns", C.c_void_p), ("act_bytes_per_sample", C.c_void_p),
                ("param_bytes", C.c_void_p), ("cut_bytes_per_sample", C.c_void_p),
                ("bandwidth_bytes_per_us", C.c_int64), ("time_bwd_per_sample_ns", C.c_void_p)]


class FormStageOut(C.Structure):
    _fields_ = [("feasible", C.c_int32), ("n", C.c_int32), ("devices", C.c_int32),
                ("replica_factor", C.c_int32), ("n_stages", C.c_int32), ("n_microbatches", C.c_int32),
                ("stage_time_ns", C.c_int64), ("est_iter_ns", C.c_int64)]


class RanncDpError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} ({status})")


_lib = None


def lib():
    """Load librannc_dp.so (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with "
                              "`python -m paper_2103_16063_amd.build` (there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        vp, sz = C.c_void_p, C.c_size_t
        L.rannc_dp_workspace_bytes.argtypes = [C.POINTER(Limits)]
        L.rannc_dp_workspace_bytes.restype = sz
        L.rannc_dp_workspace_bytes_for.argtypes = [C.POINTER(Limits), C.POINTER(Batch)]
        L.rannc_dp_workspace_bytes_for.restype = sz
        L.rannc_dp_create.argtypes = [C.POINTER(Limits), vp, sz, C.POINTER(vp)]
        L.rannc_dp_create.restype = C.c_int
        L.rannc_dp_solve.argtypes = [vp, C.POINTER(Batch), vp, vp, vp, vp, vp]
        L.rannc_dp_solve.restype = C.c_int
        L.rannc_dp_traceback.argtypes = [vp, vp, C.c_int32, vp, vp]
        L.rannc_dp_traceback.restype = C.c_int
        L.rannc_dp_read_table.argtypes = [vp, C.c_int, C.c_int32, vp, sz, vp]
        L.rannc_dp_read_table.restype = C.c_int
        L.rannc_dp_destroy.argtypes = [vp]
        L.rannc_dp_destroy.restype = None
        L.rannc_dp_strerror.argtypes = [C.c_int]
        L.rannc_dp_strerror.restype = C.c_char_p
        L.rannc_dp_set_timing.argtypes = [vp, C.c_int]
        L.rannc_dp_set_timing.restype = C.c_int
        L.rannc_dp_get_timing.argtypes = [vp, C.POINTER(C.c_float), C.POINTER(C.c_int32)]
        L.rannc_dp_get_timing.restype = C.c_int
        L.rannc_dp_traceback_at.argtypes = [vp, vp, vp, C.c_int32, vp, vp]
        L.rannc_dp_traceback_at.restype = C.c_int
        L.rannc_dp_level_values.argtypes = [vp, vp, C.c_int32, vp]
        L.rannc_dp_level_values.restype = C.c_int
        L.rannc_dp_form_stage_problems.argtypes = [C.POINTER(FormStageIn)]
        L.rannc_dp_form_stage_problems.restype = C.c_int32
        L.rannc_dp_form_stage_scratch_bytes.argtypes = [C.POINTER(FormStageIn)]
        L.rannc_dp_form_stage_scratch_bytes.restype = sz
        L.rannc_dp_form_stage.argtypes = [vp, C.POINTER(FormStageIn), vp, vp, sz,
                                          C.POINTER(FormStageOut), vp, vp, C.c_int32]
        L.rannc_dp_form_stage.restype = C.c_int
        L.rannc_dp_solve_info.argtypes = [vp, C.POINTER(SolveInfo)]
        L.rannc_dp_solve_info.restype = C.c_int
        L.rannc_dp_compact_workspace_bytes.argtypes = [C.c_int32]
        L.rannc_dp_compact_workspace_bytes.restype = sz
        L.rannc_dp_compact.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32, C.c_int64, vp, vp, vp, vp, sz, vp, vp, vp,
                                       vp, vp, vp]
        L.rannc_dp_compact.restype = C.c_int
        L.rannc_dp_compact_static.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32, C.c_int64, vp, vp, vp, vp, vp, vp,
                                              vp, vp, vp]
        L.rannc_dp_compact_static.restype = C.c_int
        _lib = L
    return _lib


def strerror(status: int) -> str:
    return lib().rannc_dp_strerror(int(status)).decode()


def _ptr(x):
    """Raw address of a torch tensor (device or host), a numpy array, an int, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if isinstance(x, np.ndarray):
        return x.ctypes.data
    return x.data_ptr()  # torch.Tensor


def make_limits(max_problems, max_blocks, max_devices, max_stages,
                max_total_time_ns=NARROW_MAX_TOTAL_TIME, algo=ALGO_AUTO, flags=0, rows_per_wave=0,
                one_launch_small=0, single_stream=0) -> Limits:
    return Limits(int(max_problems), int(max_blocks), int(max_devices), int(max_stages),
                  int(max_total_time_ns), int(algo), int(flags), int(rows_per_wave), int(one_launch_small),
                  int(single_stream), 0)


def rannc_dp_solve_info(handle):
    """Returns (status, SolveInfo)."""
    info = SolveInfo()
    rc = lib().rannc_dp_solve_info(handle, C.byref(info))
    return rc, info


class HostBatch:
    """Keeps the numpy arrays of a batch's HOST members alive next to the C struct."""

    def __init__(self, n_blocks, n_devices, max_stages, n_microbatches, mem_capacity, block_offset,
                 time_ns, param_bytes, act_bytes, bandwidth_bytes_per_us=None, cut_bytes=None,
                 time_bwd_ns=None):
        self.keep = [np.ascontiguousarray(n_blocks, dtype=np.int32),
                     np.ascontiguousarray(n_devices, dtype=np.int32),
                     np.ascontiguousarray(max_stages, dtype=np.int32),
                     np.ascontiguousarray(n_microbatches, dtype=np.int32),
                     np.ascontiguousarray(mem_capacity, dtype=np.int64),
                     np.ascontiguousarray(block_offset, dtype=np.int64)]
        self.device = (time_ns, param_bytes, act_bytes, cut_bytes, time_bwd_ns)  # DEVICE tensors (kept alive)
        self.n_problems = int(self.keep[0].shape[0])
        self.bw = (None if bandwidth_bytes_per_us is None
                   else np.ascontiguousarray(bandwidth_bytes_per_us, dtype=np.int64))
        self.struct = Batch(self.n_problems, *[_ptr(a) for a in self.keep],
                            _ptr(time_ns), _ptr(param_bytes), _ptr(act_bytes), _ptr(self.bw),
                            _ptr(cut_bytes), _ptr(time_bwd_ns))


def rannc_dp_workspace_bytes(limits: Limits) -> int:
    return int(lib().rannc_dp_workspace_bytes(C.byref(limits)))


def rannc_dp_workspace_bytes_for(limits: Limits, batch: HostBatch) -> int:
    return int(lib().rannc_dp_workspace_bytes_for(C.byref(limits), C.byref(batch.struct)))


def rannc_dp_create(limits: Limits, d_workspace, workspace_bytes: int):
    """Returns (status, handle).  d_workspace: torch uint8 tensor on the device, or an address."""
    h = C.c_void_p()
    rc = lib().rannc_dp_create(C.byref(limits), _ptr(d_workspace), int(workspace_bytes), C.byref(h))
    return rc, (h.value if rc == OK else None)


def rannc_dp_solve(handle, batch: HostBatch, stream, d_opt, d_n_stages, d_est_iter_ns=None,
                   d_status=None) -> int:
    return lib().rannc_dp_solve(handle, C.byref(batch.struct) if batch is not None else None,
                                _ptr(stream), _ptr(d_opt), _ptr(d_n_stages), _ptr(d_est_iter_ns),
                                _ptr(d_status))


def rannc_dp_traceback(handle, stream, plan_stride: int, d_stage_end, d_replicas) -> int:
    return lib().rannc_dp_traceback(handle, _ptr(stream), int(plan_stride), _ptr(d_stage_end),
                                    _ptr(d_replicas))


def rannc_dp_traceback_at(handle, stream, d_levels, plan_stride: int, d_stage_end, d_replicas) -> int:
    return lib().rannc_dp_traceback_at(handle, _ptr(stream), _ptr(d_levels), int(plan_stride),
                                       _ptr(d_stage_end), _ptr(d_replicas))


def rannc_dp_level_values(handle, stream, stride: int, d_values) -> int:
    return lib().rannc_dp_level_values(handle, _ptr(stream), int(stride), _ptr(d_values))


class HostFormStageIn:
    """Keeps the HOST arrays of a form_stage input alive next to the C struct."""

    def __init__(self, time_per_sample_ns, act_bytes_per_sample, param_bytes, n_nodes,
                 devices_per_node, batch_size, mem_capacity, cut_bytes_per_sample=None,
                 bandwidth_bytes_per_us=0, time_bwd_per_sample_ns=None):
        self.keep = [np.ascontiguousarray(time_per_sample_ns, dtype=np.int64),
                     np.ascontiguousarray(act_bytes_per_sample, dtype=np.int64),
                     np.ascontiguousarray(param_bytes, dtype=np.int64)]
        self.cut = (None if cut_bytes_per_sample is None
                    else np.ascontiguousarray(cut_bytes_per_sample, dtype=np.int64))
        self.bwd = (None if time_bwd_per_sample_ns is None
                    else np.ascontiguousarray(time_bwd_per_sample_ns, dtype=np.int64))
        self.struct = FormStageIn(int(self.keep[0].shape[0]), int(n_nodes), int(devices_per_node), 0,
                                  int(batch_size), int(mem_capacity), *[_ptr(a) for a in self.keep],
                                  _ptr(self.cut), int(bandwidth_bytes_per_us), _ptr(self.bwd))


def rannc_dp_form_stage_problems(fin: HostFormStageIn) -> int:
    return int(lib().rannc_dp_form_stage_problems(C.byref(fin.struct)))


def rannc_dp_form_stage_scratch_bytes(fin: HostFormStageIn) -> int:
    return int(lib().rannc_dp_form_stage_scratch_bytes(C.byref(fin.struct)))


def rannc_dp_form_stage(handle, fin: HostFormStageIn, stream, d_scratch, scratch_bytes: int,
                        plan_stride: int):
    """Returns (status, FormStageOut, stage_end[plan_stride], replicas[plan_stride]) (HOST arrays)."""
    out = FormStageOut()
    se = np.full(plan_stride, -2, dtype=np.int32)
    rp = np.full(plan_stride, -2, dtype=np.int32)
    rc = lib().rannc_dp_form_stage(handle, C.byref(fin.struct), _ptr(stream), _ptr(d_scratch),
                                   int(scratch_bytes), C.byref(out), _ptr(se), _ptr(rp),
                                   int(plan_stride))
    return rc, out, se, rp


def rannc_dp_compact_workspace_bytes(n_groups: int) -> int:
    return int(lib().rannc_dp_compact_workspace_bytes(int(n_groups)))


def rannc_dp_compact(stream, n_groups: int, k: int, max_walks: int, mem_capacity: int, d_time_ns, d_param_bytes,
                     d_act_bytes, d_workspace, workspace_bytes: int, d_n_blocks, d_block_end, d_time_out,
                     d_param_out, d_act_out, d_status) -> int:
    return lib().rannc_dp_compact(_ptr(stream), int(n_groups), int(k), int(max_walks), int(mem_capacity), _ptr(d_time_ns),
                                  _ptr(d_param_bytes), _ptr(d_act_bytes), _ptr(d_workspace), int(workspace_bytes),
                                  _ptr(d_n_blocks), _ptr(d_block_end), _ptr(d_time_out), _ptr(d_param_out),
                                  _ptr(d_act_out), _ptr(d_status))


COMPACT_STATIC_MAX_GROUPS = 16384


def rannc_dp_compact_static(stream, n_groups: int, k: int, max_walks: int, mem_capacity: int, d_time_ns,
                            d_param_bytes, d_act_bytes, d_n_blocks, d_block_end, d_time_out, d_param_out,
                            d_act_out, d_status) -> int:
    return lib().rannc_dp_compact_static(_ptr(stream), int(n_groups), int(k), int(max_walks), int(mem_capacity),
                                         _ptr(d_time_ns), _ptr(d_param_bytes), _ptr(d_act_bytes), _ptr(d_n_blocks),
                                         _ptr(d_block_end), _ptr(d_time_out), _ptr(d_param_out), _ptr(d_act_out),
                                         _ptr(d_status))


def rannc_dp_read_table(handle, which: int, problem: int, d_dst, nbytes: int, stream) -> int:
    return lib().rannc_dp_read_table(handle, int(which), int(problem), _ptr(d_dst), int(nbytes),
                                     _ptr(stream))


def rannc_dp_destroy(handle) -> None:
    lib().rannc_dp_destroy(handle)


def rannc_dp_set_timing(handle, enabled: bool) -> int:
    return lib().rannc_dp_set_timing(handle, 1 if enabled else 0)


def rannc_dp_get_timing(handle):
    """Returns (status, [build_ms, levels_ms, select_ms], level_launches)."""
    ms = (C.c_float * 3)()
    n = C.c_int32()
    rc = lib().rannc_dp_get_timing(handle, ms, C.byref(n))
    return rc, [float(ms[0]), float(ms[1]), float(ms[2])], int(n.value)


# ---------------------------------------------------------------------------------------------
# Convenience for tests, the smoke check and the benchmark: owns the torch buffers around one
# handle.  Still marshalling only.
# ---------------------------------------------------------------------------------------------
class Session:
    def __init__(self, batch_np: dict, *, algo=ALGO_AUTO, max_total_time_ns=NARROW_MAX_TOTAL_TIME,
                 device="cuda:0", exact_workspace=True, rows_per_wave=0, one_launch_small=0, single_stream=0):
        import torch
        self.torch = torch
        self.dev = torch.device(device)
        b = batch_np
        self.Q = int(b["n_problems"])
        self.batch_np = b
        self.S_eff = np.minimum(b["max_stages"], np.minimum(b["n_blocks"], b["n_devices"]))
        self.split = "time_bwd_ns" in b
        self.limits = make_limits(self.Q, int(b["n_blocks"].max()), int(b["n_devices"].max()),
                                  int(self.S_eff.max()), max_total_time_ns, algo,
                                  FLAG_SPLIT_OBJECTIVE if self.split else 0, rows_per_wave, one_launch_small,
                                  single_stream)
        self.d_in = [torch.from_numpy(np.ascontiguousarray(b[k], dtype=np.int64)).to(self.dev)
                     for k in ("time_ns", "param_bytes", "act_bytes")]
        self.d_bwd = None
        if self.split:
            self.d_bwd = torch.from_numpy(np.ascontiguousarray(b["time_bwd_ns"], dtype=np.int64)).to(self.dev)
        self.d_cut = None
        if "cut_bytes" in b:
            self.d_cut = torch.from_numpy(np.ascontiguousarray(b["cut_bytes"], dtype=np.int64)).to(self.dev)
        self.hb = HostBatch(b["n_blocks"], b["n_devices"], b["max_stages"], b["n_microbatches"],
                            b["mem_capacity"], b["block_offset"], *self.d_in,
                            b.get("bandwidth_bytes_per_us"), self.d_cut, self.d_bwd)
        nbytes = (rannc_dp_workspace_bytes_for(self.limits, self.hb) if exact_workspace
                  else rannc_dp_workspace_bytes(self.limits))
        if nbytes == 0:
            raise RanncDpError(INVALID_ARG, "workspace size query")
        self.ws_bytes = nbytes
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device=self.dev)
        rc, self.h = rannc_dp_create(self.limits, self.ws, nbytes)
        if rc != OK:
            raise RanncDpError(rc, "rannc_dp_create")
        self.plan_stride = int(self.S_eff.max())
        # every output of solve and traceback in ONE device buffer (and one pinned host buffer of
        # the same layout), so that the results come to the host in a single copy
        Q, PS = self.Q, self.plan_stride
        sizes = [8 * Q, 8 * Q, 4 * Q, 4 * Q, 4 * Q * PS, 4 * Q * PS]  # opt, est, n_stages, status, ends, replicas
        offs = np.concatenate(([0], np.cumsum([(x + 7) // 8 * 8 for x in sizes]))).astype(int)
        self._out_dev = torch.empty(int(offs[-1]), dtype=torch.uint8, device=self.dev)
        self._out_host = torch.empty(int(offs[-1]), dtype=torch.uint8, pin_memory=True)

        def views(buf):
            cut = lambda k, dt, shape: buf[int(offs[k]):int(offs[k]) + sizes[k]].view(dt).view(shape)
            return (cut(0, torch.int64, (Q,)), cut(1, torch.int64, (Q,)), cut(2, torch.int32, (Q,)),
                    cut(3, torch.int32, (Q,)), cut(4, torch.int32, (Q, PS)), cut(5, torch.int32, (Q, PS)))
        self.d_opt, self.d_est, self.d_ns, self.d_status, self.d_se, self.d_rp = views(self._out_dev)
        self._h_views = views(self._out_host)

    def stream(self):
        return self.torch.cuda.current_stream(self.dev).cuda_stream

    def solve(self):
        rc = rannc_dp_solve(self.h, self.hb, self.stream(), self.d_opt, self.d_ns, self.d_est,
                            self.d_status)
        if rc != OK:
            raise RanncDpError(rc, "rannc_dp_solve")

    def traceback(self):
        rc = rannc_dp_traceback(self.h, self.stream(), self.plan_stride, self.d_se, self.d_rp)
        if rc != OK:
            raise RanncDpError(rc, "rannc_dp_traceback")

    def run(self):
        """solve + traceback + ONE copy of all results to (pinned) host memory."""
        self.solve()
        self.traceback()
        self._out_host.copy_(self._out_dev, non_blocking=True)
        self.torch.cuda.current_stream(self.dev).synchronize()
        opt, est, ns, status, se, rp = (v.numpy().copy() for v in self._h_views)
        return {"opt": opt, "n_stages": ns, "est_iter_ns": est, "status": status, "stage_end": se, "replicas": rp}

    def table(self, which: int, q: int) -> np.ndarray:
        torch = self.torch
        N, D, L = (int(self.batch_np["n_blocks"][q]), int(self.batch_np["n_devices"][q]),
                   int(self.S_eff[q]))
        tri = N * (N + 1) // 2 * D
        cells = (L + 1) * (N + 1) * (D + 1)
        if which in (TABLE_COST, TABLE_COST_BWD):
            dst = torch.empty(tri, dtype=torch.int64, device=self.dev)
        elif which == TABLE_FIT:
            dst = torch.empty(tri, dtype=torch.uint8, device=self.dev)
        elif which in (TABLE_V, TABLE_MAX_FWD, TABLE_MAX_BWD):
            dst = torch.empty(cells, dtype=torch.int64, device=self.dev)
        else:
            dst = torch.empty(cells, dtype=torch.int32, device=self.dev)
        rc = rannc_dp_read_table(self.h, which, q, dst, dst.numel() * dst.element_size(),
                                 self.stream())
        if rc != OK:
            raise RanncDpError(rc, "rannc_dp_read_table")
        torch.cuda.synchronize(self.dev)
        out = dst.cpu().numpy()
        if which in (TABLE_V, TABLE_ARG_I, TABLE_ARG_D, TABLE_MAX_FWD, TABLE_MAX_BWD):
            out = out.reshape(L + 1, N + 1, D + 1)
        return out

    def close(self):
        if getattr(self, "h", None):
            self.torch.cuda.synchronize(self.dev)
            rannc_dp_destroy(self.h)
            self.h = None

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()


class FormStageSession:
    """Owns handle, workspace and scratch for rannc_dp_form_stage calls on inputs of one shape."""

    def __init__(self, n_blocks, n_nodes, devices_per_node, batch_size, *,
                 max_total_time_ns=NARROW_MAX_TOTAL_TIME, algo=ALGO_AUTO, device="cuda:0", split=False):
        import torch
        self.torch = torch
        self.dev = torch.device(device)
        self.shape = (int(n_blocks), int(n_nodes), int(devices_per_node), int(batch_size))
        probe = HostFormStageIn(np.zeros(n_blocks), np.zeros(n_blocks), np.zeros(n_blocks), n_nodes,
                                devices_per_node, batch_size, 0)
        self.Q = rannc_dp_form_stage_problems(probe)
        if self.Q == 0:
            raise RanncDpError(INVALID_ARG, "rannc_dp_form_stage_problems")
        n_max = 1
        while 2 * n_max <= n_nodes:
            n_max *= 2
        self.max_D = devices_per_node * n_max
        self.plan_stride = self.max_D
        self.limits = make_limits(self.Q, n_blocks, self.max_D, min(self.max_D, n_blocks),
                                  max_total_time_ns, algo, FLAG_SPLIT_OBJECTIVE if split else 0)
        self.ws_bytes = rannc_dp_workspace_bytes(self.limits)
        if self.ws_bytes == 0:
            raise RanncDpError(INVALID_ARG, "workspace size query")
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=self.dev)
        rc, self.h = rannc_dp_create(self.limits, self.ws, self.ws_bytes)
        if rc != OK:
            raise RanncDpError(rc, "rannc_dp_create")
        self.scratch_bytes = rannc_dp_form_stage_scratch_bytes(probe)
        self.scratch = torch.empty(self.scratch_bytes, dtype=torch.uint8, device=self.dev)

    def run(self, time_per_sample_ns, act_bytes_per_sample, param_bytes, mem_capacity,
            cut_bytes_per_sample=None, bandwidth_bytes_per_us=0, time_bwd_per_sample_ns=None):
        n_blocks, n_nodes, dn, bs = self.shape
        fin = HostFormStageIn(time_per_sample_ns, act_bytes_per_sample, param_bytes, n_nodes, dn, bs,
                              mem_capacity, cut_bytes_per_sample, bandwidth_bytes_per_us,
                              time_bwd_per_sample_ns)
        assert fin.struct.n_blocks == n_blocks
        stream = self.torch.cuda.current_stream(self.dev).cuda_stream
        return rannc_dp_form_stage(self.h, fin, stream, self.scratch, self.scratch_bytes,
                                   self.plan_stride)

    def close(self):
        if getattr(self, "h", None):
            self.torch.cuda.synchronize(self.dev)
            rannc_dp_destroy(self.h)
            self.h = None
