"""CPU checker ("oracle") -- TEST INFRASTRUCTURE, not part of the product.

Serial C++ definitions of every task kernel and a replay of the scheduler's
admission / partition policy.  Only the tests, the smoke check and the bench's
CPU-baseline leg may import this package; the GPU library never does, and this
package never imports the GPU library.
"""
import ctypes as C
import numpy as np

from .build import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build())
        _lib.orc_sched_replay.restype = C.c_int64
        _lib.orc_demand.restype = C.c_uint32
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


# ---------------------------------------------------------------- kernels
def jacobi_f64(u0, iters):
    u = np.array(u0, dtype=np.float64, order="C")
    n = u.shape[0]
    assert u.shape == (n, n)
    lib().orc_jacobi_f64(_p(u), C.c_uint32(n), C.c_uint32(iters))
    return u


def jacobi_f32(u0, iters):
    u = np.array(u0, dtype=np.float32, order="C")
    n = u.shape[0]
    assert u.shape == (n, n)
    lib().orc_jacobi_f32(_p(u), C.c_uint32(n), C.c_uint32(iters))
    return u


def gemm_f32(a, b):
    a = np.ascontiguousarray(a, dtype=np.float32)
    b = np.ascontiguousarray(b, dtype=np.float32)
    m, k = a.shape
    k2, n = b.shape
    assert k == k2
    c = np.empty((m, n), dtype=np.float64)
    lib().orc_gemm_f32(_p(a), _p(b), _p(c), C.c_uint32(m), C.c_uint32(n), C.c_uint32(k))
    return c


def gemm_abs_f32(a, b):
    a = np.ascontiguousarray(a, dtype=np.float32)
    b = np.ascontiguousarray(b, dtype=np.float32)
    m, k = a.shape
    _, n = b.shape
    c = np.empty((m, n), dtype=np.float64)
    lib().orc_gemm_abs_f32(_p(a), _p(b), _p(c), C.c_uint32(m), C.c_uint32(n), C.c_uint32(k))
    return c


def gemm_f32_entries(a, b, rows, cols):
    a = np.ascontiguousarray(a, dtype=np.float32)
    b = np.ascontiguousarray(b, dtype=np.float32)
    rows = np.ascontiguousarray(rows, dtype=np.uint32)
    cols = np.ascontiguousarray(cols, dtype=np.uint32)
    _, k = a.shape
    _, n = b.shape
    out = np.empty(rows.size, dtype=np.float64)
    out_abs = np.empty(rows.size, dtype=np.float64)
    lib().orc_gemm_f32_entries(_p(a), _p(b), C.c_uint32(n), C.c_uint32(k), _p(rows), _p(cols),
                               C.c_uint32(rows.size), _p(out), _p(out_abs))
    return out, out_abs


def gemm_bf16(a_bits, b_bits):
    a = np.ascontiguousarray(a_bits, dtype=np.uint16)
    b = np.ascontiguousarray(b_bits, dtype=np.uint16)
    m, k = a.shape
    _, n = b.shape
    c = np.empty((m, n), dtype=np.float64)
    lib().orc_gemm_bf16(_p(a), _p(b), _p(c), C.c_uint32(m), C.c_uint32(n), C.c_uint32(k))
    return c


def gemm_bf16_entries(a_bits, b_bits, rows, cols):
    a = np.ascontiguousarray(a_bits, dtype=np.uint16)
    b = np.ascontiguousarray(b_bits, dtype=np.uint16)
    rows = np.ascontiguousarray(rows, dtype=np.uint32)
    cols = np.ascontiguousarray(cols, dtype=np.uint32)
    _, k = a.shape
    _, n = b.shape
    out = np.empty(rows.size, dtype=np.float64)
    lib().orc_gemm_bf16_entries(_p(a), _p(b), C.c_uint32(n), C.c_uint32(k), _p(rows), _p(cols),
                                C.c_uint32(rows.size), _p(out))
    return out


def conv3x3_relu(x_bits, w_bits, stride):
    """x: N,H,W,C bf16 bits; w: K,3,3,C bf16 bits -> N,Ho,Wo,K float64 (after ReLU)."""
    x = np.ascontiguousarray(x_bits, dtype=np.uint16)
    w = np.ascontiguousarray(w_bits, dtype=np.uint16)
    n, h, wd, c = x.shape
    k = w.shape[0]
    assert w.shape == (k, 3, 3, c)
    ho = (h + 2 - 3) // stride + 1
    wo = (wd + 2 - 3) // stride + 1
    y = np.empty((n, ho, wo, k), dtype=np.float64)
    lib().orc_conv3x3_relu(_p(x), _p(w), _p(y), C.c_uint32(n), C.c_uint32(h), C.c_uint32(wd),
                           C.c_uint32(c), C.c_uint32(k), C.c_uint32(stride))
    return y


def round_bf16(x):
    x = np.ascontiguousarray(x, dtype=np.float64)
    out = np.empty(x.shape, dtype=np.uint16)
    lib().orc_round_bf16(_p(x), _p(out), C.c_uint64(x.size))
    return out


def cnn_forward(x_bits, weights, strides):
    """Layer chain: activations rounded to bf16 between layers, last layer kept in float64."""
    act = x_bits
    y = None
    for li, (w, s) in enumerate(zip(weights, strides)):
        y = conv3x3_relu(act, w, s)
        if li + 1 < len(weights):
            act = round_bf16(y)
    return y


def bfs(row_ptr, col_idx, source=0):
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int32)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
    n = row_ptr.size - 1
    level = np.empty(n, dtype=np.int32)
    lib().orc_bfs(_p(row_ptr), _p(col_idx), C.c_uint32(n), C.c_uint32(source), _p(level))
    return level


# ---------------------------------------------------------------- scheduler replay
class Device(C.Structure):
    _fields_ = [("cap_bytes", C.c_uint64), ("n_cu", C.c_uint32), ("granule_cus", C.c_uint32),
                ("wave_size", C.c_uint32), ("max_waves_per_cu", C.c_uint32),
                ("max_wg_per_cu", C.c_uint32), ("policy", C.c_uint32), ("queue_mode", C.c_uint32),
                ("max_running", C.c_uint32)]


INPUT_DT = np.dtype([("kind", "<u4"), ("wg_per_cu", "<u4"), ("id", "<u8"), ("mem", "<u8"),
                     ("grid", "<u4", (3,)), ("block", "<u4", (3,))])
DECISION_DT = np.dtype([("in_index", "<u4"), ("kind", "<u4"), ("ticket", "<u8"), ("task_id", "<u8"),
                        ("free_bytes", "<u8"), ("granule_mask", "<u4"), ("free_granules", "<u4"),
                        ("demand", "<u4"), ("code", "<i4"), ("cu_mask", "<u4", (8,))])

IN_PROBE, IN_COMPLETE, IN_CANCEL, IN_GROW = 0, 1, 2, 3
D_ADMIT, D_WAIT, D_REJECT, D_RELEASE, D_CANCELLED, D_GROWN = 1, 2, 3, 4, 5, 6
POL_HARD, POL_SOFT, POL_SERIAL, POL_CG = 0, 1, 2, 3
Q_BACKFILL, Q_FIFO = 0, 1


def device(cap_bytes, n_cu=256, granule_cus=8, wave_size=64, max_waves_per_cu=32,
           max_wg_per_cu=32, policy=POL_HARD, queue_mode=Q_BACKFILL, max_running=0):
    return Device(cap_bytes, n_cu, granule_cus, wave_size, max_waves_per_cu, max_wg_per_cu,
                  policy, queue_mode, max_running)


def demand(dev, grid, block, wg_per_cu=0):
    """Granules demanded by a launch geometry (and, optionally, the number of workgroups per CU
    the task's own registers / LDS allow), and its waves."""
    g = (C.c_uint32 * 3)(*grid)
    b = (C.c_uint32 * 3)(*block)
    waves = C.c_uint64(0)
    d = lib().orc_demand_ex(C.byref(dev), g, b, C.c_uint32(wg_per_cu), C.byref(waves))
    return int(d), int(waves.value)


def sched_replay(dev, inputs):
    """inputs: structured array of INPUT_DT.  Returns structured array of DECISION_DT."""
    inputs = np.ascontiguousarray(inputs, dtype=INPUT_DT)
    cap = 4 * len(inputs) + 16
    out = np.zeros(cap, dtype=DECISION_DT)
    n = lib().orc_sched_replay(C.byref(dev), _p(inputs), C.c_uint64(len(inputs)), _p(out),
                               C.c_uint64(cap))
    if n < 0:
        raise RuntimeError("decision buffer too small")
    return out[:n]


def make_inputs(events):
    """events: list of ("probe", task_id, mem, grid, block[, wg_per_cu]) | ("complete", ticket) |
    ("cancel", ticket) | ("grow", ticket, extra_bytes)."""
    arr = np.zeros(len(events), dtype=INPUT_DT)
    for i, ev in enumerate(events):
        if ev[0] == "probe":
            arr[i]["kind"] = IN_PROBE
            arr[i]["id"] = ev[1]
            arr[i]["mem"] = ev[2]
            arr[i]["grid"] = ev[3]
            arr[i]["block"] = ev[4]
            arr[i]["wg_per_cu"] = ev[5] if len(ev) > 5 else 0
        elif ev[0] == "complete":
            arr[i]["kind"] = IN_COMPLETE
            arr[i]["id"] = ev[1]
        elif ev[0] == "cancel":
            arr[i]["kind"] = IN_CANCEL
            arr[i]["id"] = ev[1]
        elif ev[0] == "grow":
            arr[i]["kind"] = IN_GROW
            arr[i]["id"] = ev[1]
            arr[i]["mem"] = ev[2]
        else:
            raise ValueError(ev[0])
    return arr
