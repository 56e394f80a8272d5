"""Task mixes: which tasks, what shapes, when they arrive.  Data only."""
from dataclasses import dataclass, field
import math
import numpy as np

from .rng import raw64, task_seed, exponential


@dataclass
class TaskSpec:
    task_id: int
    kind: str                 # "jacobi" | "gemm_f32" | "gemm_bf16" | "bfs" | "cnn"
    params: dict
    arrival_s: float
    seed: int
    extra: dict = field(default_factory=dict)


def _u(seed, i):
    return float((int(raw64(seed, np.uint64(i))) >> 11) * 2.0 ** -53)


def _arrivals(seed, n, mean_gap_s):
    gaps = exponential(seed ^ 0xA221, n, mean_gap_s)
    t = np.cumsum(gaps)
    return (t - t[0]).tolist()          # first task arrives at t = 0


def mix4(seed=1):
    """Two Jacobi 512^2 x20 and two fp32 GEMM 256^3, all at t=0, cap 1 GiB, one data seed."""
    tasks = [
        TaskSpec(0, "jacobi", dict(n=512, iters=20), 0.0, seed),
        TaskSpec(1, "gemm_f32", dict(m=256, n=256, k=256), 0.0, seed),
        TaskSpec(2, "jacobi", dict(n=512, iters=20), 0.0, seed),
        TaskSpec(3, "gemm_f32", dict(m=256, n=256, k=256), 0.0, seed),
    ]
    return dict(name="Mix-4", cap_bytes=1 << 30, tasks=tasks)


def mix16(seed=16):
    """16 tasks, exponential gaps (mean 5 ms), kind uniform over Jacobi 4096^2 x100,
    fp32 GEMM 4096^3, BFS on n=2^20 mean degree 16."""
    arr = _arrivals(seed, 16, 5e-3)
    tasks = []
    for i in range(16):
        k = int(_u(seed ^ 0xC1D, i) * 3)
        ts = task_seed(seed, i)
        if k == 0:
            tasks.append(TaskSpec(i, "jacobi", dict(n=4096, iters=100), arr[i], ts))
        elif k == 1:
            tasks.append(TaskSpec(i, "gemm_f32", dict(m=4096, n=4096, k=4096), arr[i], ts))
        else:
            tasks.append(TaskSpec(i, "bfs", dict(n=1 << 20, degree=16), arr[i], ts))
    return dict(name="Mix-16", cap_bytes=288 * 10 ** 9, tasks=tasks)


def cnn8(seed=8, h=416, w=416):
    """8 inference jobs of the 10-layer conv net, batch in {1,2,4,8}, mean gap 10 ms.
    (h, w smaller than 416 gives the reduced instances the tests recompute on the CPU.)"""
    arr = _arrivals(seed, 8, 10e-3)
    tasks = []
    for i in range(8):
        b = (1, 2, 4, 8)[int(_u(seed ^ 0xBA7C, i) * 4)]
        tasks.append(TaskSpec(i, "cnn", dict(batch=b, h=h, w=w), arr[i], task_seed(seed, i)))
    return dict(name="CNN-8", cap_bytes=288 * 10 ** 9, tasks=tasks)


def pressure32(seed=32, scale=1.0):
    """16 fp32 GEMM 32768^3 and 16 Jacobi 16384^2 x50, all at t=0.  ``scale`` < 1
    shrinks the linear sizes (multiples of 256) for tests; the cap is the summed
    footprint / 1.5 so that admission has to queue."""
    g = max(256, int(32768 * scale) // 256 * 256)
    j = max(256, int(16384 * scale) // 256 * 256)
    tasks = []
    for i in range(32):
        if i % 2 == 0:
            tasks.append(TaskSpec(i, "gemm_f32", dict(m=g, n=g, k=g), 0.0, task_seed(seed, i)))
        else:
            tasks.append(TaskSpec(i, "jacobi", dict(n=j, iters=50), 0.0, task_seed(seed, i)))
    total = 16 * 3 * g * g * 4 + 16 * 2 * j * j * 4
    return dict(name="Pressure-32", cap_bytes=int(total / 1.5), tasks=tasks)


def kinds5(seed=5):
    """One task of every kind at its full size, all at t=0: Jacobi 4096^2 x100, fp32 GEMM 4096^3,
    bf16 GEMM 8192^3, the conv net on a batch of 8, BFS on 2^20 vertices.  Not one of the paper's
    mixes: run serialised, it gives every kernel's time alone on the device."""
    tasks = [
        TaskSpec(0, "jacobi", dict(n=4096, iters=100), 0.0, task_seed(seed, 0)),
        TaskSpec(1, "gemm_f32", dict(m=4096, n=4096, k=4096), 0.0, task_seed(seed, 1)),
        TaskSpec(2, "gemm_bf16", dict(m=8192, n=8192, k=8192), 0.0, task_seed(seed, 2)),
        TaskSpec(3, "cnn", dict(batch=8, h=416, w=416), 0.0, task_seed(seed, 3)),
        TaskSpec(4, "bfs", dict(n=1 << 20, degree=16), 0.0, task_seed(seed, 4)),
    ]
    return dict(name="Kinds-5", cap_bytes=288 * 10 ** 9, tasks=tasks)


def _logu(u, lo, hi):
    return math.exp(math.log(lo) + u * (math.log(hi) - math.log(lo)))


def mixed128(seed=128, n_tasks=128, shrink=1):
    """128 tasks, mean gap 2 ms, log-uniform sizes rounded to multiples of 64.
    shrink > 1 divides the linear sizes (and BFS vertex counts by shrink^2) for CPU-checkable runs."""
    arr = _arrivals(seed, n_tasks, 2e-3)
    tasks = []
    for i in range(n_tasks):
        k = int(_u(seed ^ 0xC1D, i) * 3)
        u1 = _u(seed ^ 0x51, i)
        u2 = _u(seed ^ 0x52, i)
        ts = task_seed(seed, i)
        if k == 0:
            n = max(64, int(round(_logu(u1, 1024, 8192) / shrink / 64)) * 64)
            tasks.append(TaskSpec(i, "jacobi", dict(n=n, iters=50), arr[i], ts))
        elif k == 1:
            n = max(64, int(round(_logu(u1, 1024, 8192) / shrink / 64)) * 64)
            kind = "gemm_f32" if u2 < 0.5 else "gemm_bf16"
            tasks.append(TaskSpec(i, kind, dict(m=n, n=n, k=n), arr[i], ts))
        else:
            n = max(64, int(round(_logu(u1, 1 << 16, 1 << 22) / (shrink * shrink))))
            d = int(round(_logu(u2, 8, 32)))
            tasks.append(TaskSpec(i, "bfs", dict(n=n, degree=d), arr[i], ts))
    return dict(name="Mixed-128", cap_bytes=288 * 10 ** 9, tasks=tasks)


MIXES = {"mix4": mix4, "mix16": mix16, "cnn8": cnn8, "pressure32": pressure32,
         "mixed128": mixed128, "kinds5": kinds5}
