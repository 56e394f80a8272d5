"""ctypes declarations mirroring include/mgb.h, plus small marshalling helpers."""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmgb.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "libmgb.so is not built: run `python -m paper_2107_08538_amd.build` "
        "(or __graft_entry__.build()) first; there is no fallback path")

# PyTorch provides device memory and streams, and it bundles its own copy of the
# HIP runtime (same soname as the one libmgb.so was linked against).  A process
# must hold exactly one HIP runtime, so torch is loaded first and libmgb.so then
# binds to that copy; loading them the other way round gives two runtimes of
# which the second finds no device.
import torch  # noqa: E402,F401

lib = C.CDLL(LIB_PATH)

MGB_OK, MGB_WAIT, MGB_TIMEOUT = 0, 1, 2
MGB_E_INVAL, MGB_E_TOO_BIG, MGB_E_UNKNOWN_TICKET, MGB_E_BAD_STATE = -1, -2, -3, -4
MGB_E_BUSY, MGB_E_BACKEND, MGB_E_UNSUPPORTED, MGB_E_OOM = -5, -6, -7, -8
MGB_POLICY_HARD, MGB_POLICY_SOFT, MGB_POLICY_SERIAL, MGB_POLICY_CG = 0, 1, 2, 3
MGB_QUEUE_BACKFILL, MGB_QUEUE_FIFO = 0, 1
MGB_BACKEND_NULL, MGB_BACKEND_HIP = 0, 1
MGB_EV_PROBE, MGB_EV_COMPLETE, MGB_EV_CANCEL, MGB_EV_GROW = 0, 1, 2, 3
MGB_EV_ADMIT, MGB_EV_QUEUED, MGB_EV_REJECT, MGB_EV_RELEASE, MGB_EV_CANCELLED, MGB_EV_GROWN = 16, 17, 18, 19, 20, 21


class mgb_dim3(C.Structure):
    _fields_ = [("x", C.c_uint32), ("y", C.c_uint32), ("z", C.c_uint32)]

    def tuple(self):
        return (self.x, self.y, self.z)


class mgb_device_desc(C.Structure):
    _fields_ = [("mem_cap_bytes", C.c_uint64), ("n_cu", C.c_uint32), ("granule_cus", C.c_uint32),
                ("wave_size", C.c_uint32), ("max_waves_per_cu", C.c_uint32),
                ("max_wg_per_cu", C.c_uint32), ("policy", C.c_uint32), ("queue_mode", C.c_uint32),
                ("backend", C.c_uint32), ("device", C.c_int32), ("max_running", C.c_uint32)]


class mgb_placement(C.Structure):
    _fields_ = [("ticket", C.c_uint64), ("granule_mask", C.c_uint32), ("n_granules", C.c_uint32),
                ("cu_mask", C.c_uint32 * 8), ("stream", C.c_void_p)]


class mgb_stats(C.Structure):
    _fields_ = [("free_bytes", C.c_uint64), ("free_granules", C.c_uint32),
                ("n_running", C.c_uint32), ("n_waiting", C.c_uint32), ("n_streams", C.c_uint32),
                ("n_events", C.c_uint64)]


class mgb_task_record(C.Structure):
    _fields_ = [("ticket", C.c_uint64), ("task_id", C.c_uint64), ("mem_bytes", C.c_uint64),
                ("probe_ns", C.c_uint64), ("admit_ns", C.c_uint64), ("release_ns", C.c_uint64),
                ("done_ns", C.c_uint64), ("gpu_ms", C.c_double), ("gpu_start_ms", C.c_double),
                ("gpu_stop_ms", C.c_double), ("granule_mask", C.c_uint32), ("demand", C.c_uint32),
                ("status", C.c_int32), ("reserved", C.c_uint32)]


class mgb_summary(C.Structure):
    _fields_ = [("n_done", C.c_uint64), ("n_crashed", C.c_uint64), ("n_unfinished", C.c_uint64),
                ("tasks_per_s", C.c_double), ("makespan_ms", C.c_double),
                ("mean_turnaround_ms", C.c_double), ("max_turnaround_ms", C.c_double),
                ("mean_wait_ms", C.c_double), ("max_wait_ms", C.c_double), ("gpu_busy_ms", C.c_double),
                ("max_slowdown", C.c_double), ("mean_slowdown", C.c_double)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


class mgb_conv_layer(C.Structure):
    _fields_ = [("c_in", C.c_uint32), ("c_out", C.c_uint32), ("stride", C.c_uint32)]


class mgb_task_desc(C.Structure):
    _fields_ = [("kind", C.c_uint32), ("reserved", C.c_uint32), ("task_id", C.c_uint64),
                ("arrival_ns", C.c_uint64), ("count", C.c_uint64), ("ptr", C.c_void_p * 4),
                ("dim", C.c_uint32 * 4), ("layers", C.POINTER(mgb_conv_layer)),
                ("weights", C.POINTER(C.c_void_p))]


class mgb_pool_result(C.Structure):
    _fields_ = [("status", C.c_int32), ("aux", C.c_uint32), ("ticket", C.c_uint64),
                ("arrival_ns", C.c_uint64), ("record", mgb_task_record)]


MGB_TASK_JACOBI, MGB_TASK_GEMM_F32, MGB_TASK_GEMM_BF16, MGB_TASK_BFS, MGB_TASK_CNN, MGB_TASK_CUSTOM = range(6)
MGB_POOL_ARRIVALS, MGB_POOL_RELEASE_ON_STREAM = 1, 2

TRACE_DT = np.dtype([("seq", "<u8"), ("t_ns", "<u8"), ("task_id", "<u8"), ("ticket", "<u8"),
                     ("mem_bytes", "<u8"), ("free_bytes", "<u8"), ("kind", "<u4"), ("code", "<i4"),
                     ("granule_mask", "<u4"), ("free_granules", "<u4"), ("demand", "<u4"),
                     ("cause_seq", "<u4"), ("grid", "<u4", (3,)), ("block", "<u4", (3,)),
                     ("cu_mask", "<u4", (8,))])
assert TRACE_DT.itemsize == 128

ENQUEUE_FN = C.CFUNCTYPE(C.c_int, C.c_void_p, C.c_void_p)

_u32, _u64, _vp, _i64 = C.c_uint32, C.c_uint64, C.c_void_p, C.c_int64
_P = C.POINTER


def _sig(name, restype, *argtypes):
    fn = getattr(lib, name)       # AttributeError here = header / library mismatch
    fn.restype = restype
    fn.argtypes = list(argtypes)
    return fn


mgb_device_desc_default = _sig("mgb_device_desc_default", None, _P(mgb_device_desc))
mgb_sched_create = _sig("mgb_sched_create", C.c_int, _P(mgb_device_desc), _P(_vp))
mgb_sched_destroy = _sig("mgb_sched_destroy", C.c_int, _vp)
mgb_task_probe = _sig("mgb_task_probe", C.c_int, _vp, _u64, _u64, mgb_dim3, mgb_dim3, _P(mgb_placement))
mgb_task_probe_ex = _sig("mgb_task_probe_ex", C.c_int, _vp, _u64, _u64, mgb_dim3, mgb_dim3, _u32, _P(mgb_placement))
mgb_task_wait = _sig("mgb_task_wait", C.c_int, _vp, _u64, _i64, _P(mgb_placement))
mgb_task_cancel = _sig("mgb_task_cancel", C.c_int, _vp, _u64)
mgb_task_grow = _sig("mgb_task_grow", C.c_int, _vp, _u64, _u64)


class mgb_lazy_stats(C.Structure):
    _fields_ = [("n_objects", C.c_uint64), ("n_bound", C.c_uint64), ("n_tasks", C.c_uint64),
                ("recorded_ops", C.c_uint64), ("replayed_ops", C.c_uint64), ("staged_bytes", C.c_uint64)]


mgb_lazy_create = _sig("mgb_lazy_create", C.c_int, _vp, C.POINTER(C.c_void_p))
mgb_lazy_destroy = _sig("mgb_lazy_destroy", C.c_int, _vp)
mgb_lazy_malloc = _sig("mgb_lazy_malloc", C.c_int, _vp, _u64, C.POINTER(C.c_uint64))
mgb_lazy_memcpy_h2d = _sig("mgb_lazy_memcpy_h2d", C.c_int, _vp, _u64, _vp, _u64)
mgb_lazy_memset = _sig("mgb_lazy_memset", C.c_int, _vp, _u64, C.c_int, _u64)
mgb_lazy_launch_prepare = _sig("mgb_lazy_launch_prepare", C.c_int, _vp, _u64, C.POINTER(C.c_uint64), _u32,
                               mgb_dim3, mgb_dim3, _u32, C.c_int64, C.POINTER(C.c_void_p), C.POINTER(mgb_placement))
mgb_lazy_memcpy_d2h = _sig("mgb_lazy_memcpy_d2h", C.c_int, _vp, _vp, _u64, _u64)
mgb_lazy_free = _sig("mgb_lazy_free", C.c_int, _vp, _u64)
mgb_lazy_stats_get = _sig("mgb_lazy_stats_get", C.c_int, _vp, C.POINTER(mgb_lazy_stats))
mgb_task_launch = _sig("mgb_task_launch", C.c_int, _vp, _u64, ENQUEUE_FN, _vp)
mgb_task_sync = _sig("mgb_task_sync", C.c_int, _vp, _u64, _P(C.c_double))
mgb_task_complete = _sig("mgb_task_complete", C.c_int, _vp, _u64)
mgb_task_complete_on_stream = _sig("mgb_task_complete_on_stream", C.c_int, _vp, _u64)
mgb_task_deps = _sig("mgb_task_deps", C.c_int64, _vp, _u64, _P(_u64), _u64)
mgb_task_records = _sig("mgb_task_records", C.c_int64, _vp, _u64, _P(mgb_task_record), _u64)
mgb_pool_run = _sig("mgb_pool_run", C.c_int, _vp, _P(mgb_task_desc), _u32, _u32, _u32, _P(mgb_pool_result), _P(_u64))
mgb_accounting = _sig("mgb_accounting", C.c_int, _P(mgb_task_record), _u64, _P(_u64), _P(C.c_double), _P(mgb_summary))
mgb_sched_stats = _sig("mgb_sched_stats", C.c_int, _vp, _P(mgb_stats))
mgb_trace_read = _sig("mgb_trace_read", _i64, _vp, _u64, _vp, _u64)
mgb_trace_dump = _sig("mgb_trace_dump", C.c_int, _vp, C.c_char_p)
mgb_last_error = _sig("mgb_last_error", C.c_char_p)

_probe_tail = (_P(_u64), _P(mgb_dim3), _P(mgb_dim3))
mgb_jacobi_probe = _sig("mgb_jacobi_probe", C.c_int, _u32, _u32, *_probe_tail)
mgb_jacobi_enqueue = _sig("mgb_jacobi_enqueue", C.c_int, _vp, _vp, _vp, _u32, _u32)
mgb_jacobi_launch_count = _sig("mgb_jacobi_launch_count", _u32, _u32, _u32)
mgb_jacobi_residency = _sig("mgb_jacobi_residency", _u32, _u32)
mgb_gemm_f32_residency = _sig("mgb_gemm_f32_residency", _u32, _u32, _u32, _u32)
mgb_gemm_bf16_residency = _sig("mgb_gemm_bf16_residency", _u32, _u32, _u32, _u32)
mgb_conv3x3_residency = _sig("mgb_conv3x3_residency", _u32, _u32, _u32, _u32, _u32, _u32, _u32)
mgb_cnn_residency = _sig("mgb_cnn_residency", _u32, _P(mgb_conv_layer), _u32, _u32, _u32, _u32)
mgb_bfs_residency = _sig("mgb_bfs_residency", _u32, _u32)
mgb_gemm_f32_probe = _sig("mgb_gemm_f32_probe", C.c_int, _u32, _u32, _u32, *_probe_tail)
mgb_gemm_f32_enqueue = _sig("mgb_gemm_f32_enqueue", C.c_int, _vp, _vp, _vp, _vp, _u32, _u32, _u32)
mgb_gemm_bf16_probe = _sig("mgb_gemm_bf16_probe", C.c_int, _u32, _u32, _u32, *_probe_tail)
mgb_gemm_bf16_enqueue = _sig("mgb_gemm_bf16_enqueue", C.c_int, _vp, _vp, _vp, _vp, _u32, _u32, _u32)
mgb_conv3x3_probe = _sig("mgb_conv3x3_probe", C.c_int, _u32, _u32, _u32, _u32, _u32, _u32, *_probe_tail)
mgb_conv3x3_enqueue = _sig("mgb_conv3x3_enqueue", C.c_int, _vp, _vp, _vp, _vp, _u32, _u32, _u32,
                           _u32, _u32, _u32, _u32)
mgb_cnn_probe = _sig("mgb_cnn_probe", C.c_int, _P(mgb_conv_layer), _u32, _u32, _u32, _u32,
                     _P(_u64), _P(_u64), _P(_u64), _P(mgb_dim3), _P(mgb_dim3))
mgb_cnn_enqueue = _sig("mgb_cnn_enqueue", C.c_int, _vp, _P(mgb_conv_layer), _u32, _vp, _P(_vp),
                       _vp, _vp, _vp, _u32, _u32, _u32)
mgb_bfs_work_bytes = _sig("mgb_bfs_work_bytes", _u64, _u32)
mgb_bfs_probe = _sig("mgb_bfs_probe", C.c_int, _u32, _u64, *_probe_tail)
mgb_bfs_enqueue = _sig("mgb_bfs_enqueue", C.c_int, _vp, _vp, _vp, _u32, _u32, _vp, _vp, _P(_u32))
mgb_bfs_directed_enqueue = _sig("mgb_bfs_directed_enqueue", C.c_int, _vp, _vp, _vp, _u32, _u32, _vp, _vp, _P(_u32))
mgb_bfs_enqueue_static = _sig("mgb_bfs_enqueue_static", C.c_int, _vp, _vp, _vp, _u32, _u32, _vp, _P(_u32))
mgb_cu_trace_enqueue = _sig("mgb_cu_trace_enqueue", C.c_int, _vp, _vp, _u32)
mgb_copy_enqueue = _sig("mgb_copy_enqueue", C.c_int, _vp, _vp, _vp, _u64)
mgb_mfma_loop_enqueue = _sig("mgb_mfma_loop_enqueue", C.c_int, _vp, _u32, _u32, _u32, _vp, _P(C.c_double))
mgb_fetch_rate_enqueue = _sig("mgb_fetch_rate_enqueue", C.c_int, _vp, _vp, _u64, _u32, _u32, _u32, _u32, _vp, _P(C.c_double))
mgb_lds_read_rate_enqueue = _sig("mgb_lds_read_rate_enqueue", C.c_int, _vp, _u32, _u32, _u32, _vp, _P(C.c_double))

EXPORTS = [
    "mgb_device_desc_default", "mgb_sched_create", "mgb_sched_destroy", "mgb_task_probe",
    "mgb_task_probe_ex", "mgb_gemm_f32_residency", "mgb_gemm_bf16_residency", "mgb_conv3x3_residency",
    "mgb_cnn_residency", "mgb_bfs_residency", "mgb_task_wait", "mgb_task_cancel", "mgb_task_grow", "mgb_lazy_create", "mgb_lazy_destroy", "mgb_lazy_malloc",
    "mgb_lazy_memcpy_h2d", "mgb_lazy_memset", "mgb_lazy_launch_prepare", "mgb_lazy_memcpy_d2h", "mgb_lazy_free",
    "mgb_lazy_stats_get", "mgb_server_start", "mgb_server_stop", "mgb_server_reclaimed", "mgb_client_connect",
    "mgb_client_disconnect", "mgb_client_probe", "mgb_client_wait", "mgb_client_cancel", "mgb_client_grow",
    "mgb_client_complete", "mgb_client_stats", "mgb_client_stream", "mgb_task_launch", "mgb_task_sync", "mgb_task_complete",
    "mgb_task_complete_on_stream", "mgb_task_deps", "mgb_task_records", "mgb_accounting", "mgb_pool_run",
    "mgb_sched_stats", "mgb_trace_read", "mgb_trace_dump", "mgb_last_error",
    "mgb_jacobi_probe", "mgb_jacobi_enqueue", "mgb_jacobi_launch_count", "mgb_gemm_f32_probe", "mgb_gemm_f32_enqueue",
    "mgb_gemm_bf16_probe", "mgb_gemm_bf16_enqueue", "mgb_conv3x3_probe", "mgb_conv3x3_enqueue",
    "mgb_cnn_probe", "mgb_cnn_enqueue", "mgb_bfs_work_bytes", "mgb_bfs_probe", "mgb_bfs_enqueue", "mgb_bfs_directed_enqueue", "mgb_bfs_enqueue_static",
    "mgb_cu_trace_enqueue", "mgb_copy_enqueue", "mgb_mfma_loop_enqueue", "mgb_fetch_rate_enqueue", "mgb_lds_read_rate_enqueue", "mgb_jacobi_residency",
]


# ------------------------------------------------------------------ helpers
class MgbError(RuntimeError):
    def __init__(self, code, where):
        msg = mgb_last_error().decode() if code == MGB_E_BACKEND else ""
        super().__init__("%s failed with status %d %s" % (where, code, msg))
        self.code = code


def check(code, where):
    if code < 0:
        raise MgbError(code, where)
    return code


def default_desc(**overrides):
    d = mgb_device_desc()
    mgb_device_desc_default(C.byref(d))
    for k, v in overrides.items():
        setattr(d, k, v)
    return d


def dev_ptr(t):
    """Device address of a torch tensor (or None)."""
    return None if t is None else C.c_void_p(t.data_ptr())


def probe_of(fn, *shape):
    """Call one of the mgb_*_probe functions; returns (mem_bytes, grid, block)."""
    mem, grid, block = _u64(0), mgb_dim3(), mgb_dim3()
    check(fn(*shape, C.byref(mem), C.byref(grid), C.byref(block)), fn.__name__)
    return int(mem.value), grid, block


mgb_server_start = _sig("mgb_server_start", C.c_int, _vp, C.c_char_p, _u32, C.POINTER(C.c_void_p))
mgb_server_stop = _sig("mgb_server_stop", C.c_int, _vp)
mgb_server_reclaimed = _sig("mgb_server_reclaimed", C.c_uint64, _vp)
mgb_client_connect = _sig("mgb_client_connect", C.c_int, C.c_char_p, C.POINTER(C.c_void_p))
mgb_client_disconnect = _sig("mgb_client_disconnect", C.c_int, _vp)
mgb_client_probe = _sig("mgb_client_probe", C.c_int, _vp, _u64, _u64, mgb_dim3, mgb_dim3, _u32, C.POINTER(mgb_placement))
mgb_client_wait = _sig("mgb_client_wait", C.c_int, _vp, _u64, C.c_int64, C.POINTER(mgb_placement))
mgb_client_cancel = _sig("mgb_client_cancel", C.c_int, _vp, _u64)
mgb_client_grow = _sig("mgb_client_grow", C.c_int, _vp, _u64, _u64)
mgb_client_complete = _sig("mgb_client_complete", C.c_int, _vp, _u64)
mgb_client_stats = _sig("mgb_client_stats", C.c_int, _vp, C.POINTER(mgb_stats))
mgb_client_stream = _sig("mgb_client_stream", C.c_int, _vp, C.POINTER(mgb_placement), C.POINTER(C.c_void_p))


class Server:
    """Publishes a scheduler to other processes; methods are 1:1 with the C entry points."""

    def __init__(self, sched, name, n_slots=16):
        h = _vp()
        check(mgb_server_start(sched.h, name.encode(), n_slots, C.byref(h)), "mgb_server_start")
        self.h = h

    def reclaimed(self):
        return int(mgb_server_reclaimed(self.h))

    def stop(self):
        rc = mgb_server_stop(self.h)
        self.h = None
        return rc


class Client:
    """One connection to a published scheduler; methods are 1:1 with the C entry points."""

    def __init__(self, name):
        h = _vp()
        check(mgb_client_connect(name.encode(), C.byref(h)), "mgb_client_connect")
        self.h = h

    def probe(self, task_id, mem_bytes, grid, block, wg_per_cu=0):
        grid = grid if isinstance(grid, mgb_dim3) else mgb_dim3(*grid)
        block = block if isinstance(block, mgb_dim3) else mgb_dim3(*block)
        pl = mgb_placement()
        rc = mgb_client_probe(self.h, task_id, mem_bytes, grid, block, wg_per_cu, C.byref(pl))
        return rc, pl

    def wait(self, ticket, timeout_ns=-1):
        pl = mgb_placement()
        rc = mgb_client_wait(self.h, ticket, timeout_ns, C.byref(pl))
        return rc, pl

    def cancel(self, ticket):
        return mgb_client_cancel(self.h, ticket)

    def grow(self, ticket, extra_bytes):
        return mgb_client_grow(self.h, ticket, extra_bytes)

    def complete(self, ticket):
        return mgb_client_complete(self.h, ticket)

    def stats(self):
        st = mgb_stats()
        check(mgb_client_stats(self.h, C.byref(st)), "mgb_client_stats")
        return st

    def stream(self, placement):
        st = C.c_void_p()
        rc = mgb_client_stream(self.h, C.byref(placement), C.byref(st))
        return rc, st

    def disconnect(self):
        rc = mgb_client_disconnect(self.h)
        if rc == MGB_OK:
            self.h = None
        return rc


class Lazy:
    """Owns one mgb_lazy handle; methods are 1:1 with the C entry points."""

    def __init__(self, sched):
        h = _vp()
        check(mgb_lazy_create(sched.h, C.byref(h)), "mgb_lazy_create")
        self.h = h

    def malloc(self, nbytes):
        p = C.c_uint64()
        rc = mgb_lazy_malloc(self.h, nbytes, C.byref(p))
        return rc, p.value

    def memcpy_h2d(self, dst_pseudo, host_ptr, nbytes):
        return mgb_lazy_memcpy_h2d(self.h, dst_pseudo, host_ptr, nbytes)

    def memset(self, dst_pseudo, value, nbytes):
        return mgb_lazy_memset(self.h, dst_pseudo, value, nbytes)

    def launch_prepare(self, task_id, pseudo_args, grid, block, timeout_ns=-1, wg_per_cu=0):
        n = len(pseudo_args)
        args = (C.c_uint64 * n)(*pseudo_args)
        real = (C.c_void_p * n)()
        pl = mgb_placement()
        grid = grid if isinstance(grid, mgb_dim3) else mgb_dim3(*grid)
        block = block if isinstance(block, mgb_dim3) else mgb_dim3(*block)
        rc = mgb_lazy_launch_prepare(self.h, task_id, args, n, grid, block, wg_per_cu, timeout_ns, real, C.byref(pl))
        return rc, [int(x or 0) for x in real], pl

    def memcpy_d2h(self, host_ptr, src_pseudo, nbytes):
        return mgb_lazy_memcpy_d2h(self.h, host_ptr, src_pseudo, nbytes)

    def free(self, pseudo):
        return mgb_lazy_free(self.h, pseudo)

    def stats(self):
        st = mgb_lazy_stats()
        check(mgb_lazy_stats_get(self.h, C.byref(st)), "mgb_lazy_stats_get")
        return st

    def destroy(self):
        rc = mgb_lazy_destroy(self.h)
        if rc == MGB_OK:
            self.h = None
        return rc


class Sched:
    """Owns one mgb_sched handle; methods are 1:1 with the C entry points."""

    def __init__(self, desc=None, **overrides):
        self.desc = desc if desc is not None else default_desc(**overrides)
        h = _vp()
        check(mgb_sched_create(C.byref(self.desc), C.byref(h)), "mgb_sched_create")
        self.h = h

    def probe(self, task_id, mem_bytes, grid, block, wg_per_cu=0):
        grid = grid if isinstance(grid, mgb_dim3) else mgb_dim3(*grid)
        block = block if isinstance(block, mgb_dim3) else mgb_dim3(*block)
        pl = mgb_placement()
        if wg_per_cu:
            rc = mgb_task_probe_ex(self.h, task_id, mem_bytes, grid, block, wg_per_cu, C.byref(pl))
        else:
            rc = mgb_task_probe(self.h, task_id, mem_bytes, grid, block, C.byref(pl))
        return rc, pl

    def wait(self, ticket, timeout_ns=-1):
        pl = mgb_placement()
        rc = mgb_task_wait(self.h, ticket, timeout_ns, C.byref(pl))
        return rc, pl

    def cancel(self, ticket):
        return mgb_task_cancel(self.h, ticket)

    def grow(self, ticket, extra_bytes):
        return mgb_task_grow(self.h, ticket, extra_bytes)

    def launch(self, ticket, fn):
        """fn(stream_void_p) -> int enqueues the task's kernels."""
        cb = ENQUEUE_FN(lambda stream, user: int(fn(stream) or 0))
        return mgb_task_launch(self.h, ticket, cb, None)

    def sync(self, ticket):
        ms = C.c_double(0.0)
        rc = mgb_task_sync(self.h, ticket, C.byref(ms))
        return rc, ms.value

    def complete(self, ticket):
        return mgb_task_complete(self.h, ticket)

    def complete_on_stream(self, ticket):
        return mgb_task_complete_on_stream(self.h, ticket)

    def deps(self, ticket):
        out = (_u64 * 64)()
        n = int(mgb_task_deps(self.h, ticket, out, 64))
        check(n, "mgb_task_deps")
        return [int(out[i]) for i in range(min(n, 64))]

    def records(self, first_ticket=1, cap=1 << 16):
        out = (mgb_task_record * cap)()
        n = int(mgb_task_records(self.h, first_ticket, out, cap))
        check(n, "mgb_task_records")
        return out, n

    def stats(self):
        st = mgb_stats()
        check(mgb_sched_stats(self.h, C.byref(st)), "mgb_sched_stats")
        return st

    def trace(self):
        n = int(self.stats().n_events)
        out = np.zeros(n, dtype=TRACE_DT)
        got = mgb_trace_read(self.h, 0, out.ctypes.data_as(_vp), n)
        check(int(got), "mgb_trace_read")
        return out[:got]

    def dump(self, path):
        return mgb_trace_dump(self.h, path.encode())

    def destroy(self):
        if self.h is not None:
            rc = mgb_sched_destroy(self.h)
            if rc == MGB_OK:
                self.h = None
            return rc
        return MGB_OK


__all__ = [n for n in dir() if n.startswith(("mgb_", "MGB_"))] + [
    "lib", "LIB_PATH", "TRACE_DT", "ENQUEUE_FN", "EXPORTS", "MgbError", "check", "default_desc",
    "dev_ptr", "probe_of", "Sched", "Lazy", "Server", "Client"]
