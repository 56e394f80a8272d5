"""Worker-pool harness that pushes a task mix through the scheduler (Sec. V-A of the paper: a pool
of workers, each taking a job, running it and pulling the next; jobs either all queued at t = 0 or
arriving over time).  Pure orchestration: every call below is one C-ABI entry point."""
import ctypes as C
import threading
import time

import torch

from . import binding as mgb


def _ptr(t):
    return C.c_void_p(t.data_ptr())


class Task:
    """Device-resident buffers of one task plus its probe (footprint and geometry)."""

    def __init__(self, spec, tensors, probe, enqueue, kernel_name, launches, alg_bytes=0.0, alg_flops=0.0,
                 wg_per_cu=0):
        self.wg_per_cu = wg_per_cu      # workgroups per CU the kernel's registers and LDS allow (0: not known)
        self.spec = spec
        self.tensors = tensors          # keeps the device buffers alive
        self.mem, self.grid, self.block = probe
        self.enqueue = enqueue          # fn(stream) -> status
        self.kernel_name = kernel_name
        self.launches = launches        # kernel launches per task (None if data dependent)
        self.alg_bytes = alg_bytes      # algorithmic HBM bytes of the whole task
        self.alg_flops = alg_flops
        self.edges = 0                  # stored (directed) edges of a graph task


def build_task(spec, data, device="cuda:0"):
    """Upload one task's inputs (numpy arrays from the workload generators) and bind its entry points."""
    k, p = spec.kind, spec.params
    if k == "jacobi":
        n, it = p["n"], p["iters"]
        u0 = torch.from_numpy(data["u"]).to(device)
        u1 = u0.clone()
        probe = mgb.probe_of(mgb.mgb_jacobi_probe, n, it)
        fn = lambda st: mgb.mgb_jacobi_enqueue(st, _ptr(u0), _ptr(u1), n, it)
        # launches of five to eight sweeps (grids of 4096 columns and more) are the streaming kernel
        name = "jacobi_stream" if n >= 4096 and n % 4 == 0 and it >= 5 else "jacobi_sweeps"
        return Task(spec, dict(u0=u0, u1=u1), probe, fn, name, int(mgb.mgb_jacobi_launch_count(n, it)),
                    alg_bytes=8.0 * (n - 2) * (n - 2) * it, alg_flops=4.0 * (n - 2) * (n - 2) * it,
                    wg_per_cu=int(mgb.mgb_jacobi_residency(n)))
    if k == "gemm_f32":
        m, n, kk = p["m"], p["n"], p["k"]
        A, B = torch.from_numpy(data["a"]).to(device), torch.from_numpy(data["b"]).to(device)
        Cc = torch.zeros(m, n, device=device)
        probe = mgb.probe_of(mgb.mgb_gemm_f32_probe, m, n, kk)
        fn = lambda st: mgb.mgb_gemm_f32_enqueue(st, _ptr(A), _ptr(B), _ptr(Cc), m, n, kk)
        return Task(spec, dict(A=A, B=B, C=Cc), probe, fn, "gemm_f32_dma_kernel", 1,
                    alg_bytes=4.0 * (m * kk + kk * n + m * n), alg_flops=2.0 * m * n * kk,
                    wg_per_cu=int(mgb.mgb_gemm_f32_residency(m, n, kk)))
    if k == "gemm_bf16":
        m, n, kk = p["m"], p["n"], p["k"]
        A = torch.from_numpy(data["a"].view("int16")).to(device)
        B = torch.from_numpy(data["b"].view("int16")).to(device)
        Cc = torch.zeros(m, n, device=device)
        probe = mgb.probe_of(mgb.mgb_gemm_bf16_probe, m, n, kk)
        fn = lambda st: mgb.mgb_gemm_bf16_enqueue(st, _ptr(A), _ptr(B), _ptr(Cc), m, n, kk)
        return Task(spec, dict(A=A, B=B, C=Cc), probe, fn, "gemm_bf16_dma_kernel", 1,
                    alg_bytes=2.0 * (m * kk + kk * n) + 4.0 * m * n, alg_flops=2.0 * m * n * kk,
                    wg_per_cu=int(mgb.mgb_gemm_bf16_residency(m, n, kk)))
    if k == "bfs":
        n = p["n"]
        rp = torch.from_numpy(data["row_ptr"]).to(device)
        ci = torch.from_numpy(data["col_idx"]).to(device)
        m_edges = int(data["col_idx"].size)
        level = torch.empty(n, dtype=torch.int32, device=device)
        work = torch.zeros(mgb.mgb_bfs_work_bytes(n), dtype=torch.uint8, device=device)
        probe = mgb.probe_of(mgb.mgb_bfs_probe, n, m_edges)
        depth = C.c_uint32(0)
        fn = lambda st: mgb.mgb_bfs_enqueue(st, _ptr(rp), _ptr(ci), n, 0, _ptr(level), _ptr(work), C.byref(depth))
        t = Task(spec, dict(rp=rp, ci=ci, level=level, work=work), probe, fn, "bfs_level", None,
                 alg_bytes=8.0 * m_edges + 24.0 * n, wg_per_cu=int(mgb.mgb_bfs_residency(n)))
        t.depth = depth
        t.edges = m_edges
        return t
    if k == "cnn":
        layers = data["layers"]
        arr = (mgb.mgb_conv_layer * len(layers))(*[mgb.mgb_conv_layer(L["c_in"], L["c_out"], L["stride"]) for L in layers])
        b, h, w = p["batch"], p["h"], p["w"]
        mem, act, ob = C.c_uint64(), C.c_uint64(), C.c_uint64()
        g, blk = mgb.mgb_dim3(), mgb.mgb_dim3()
        mgb.check(mgb.mgb_cnn_probe(arr, len(layers), b, h, w, C.byref(mem), C.byref(act), C.byref(ob),
                                    C.byref(g), C.byref(blk)), "mgb_cnn_probe")
        X = torch.from_numpy(data["x"].view("int16")).to(device)
        Wd = [torch.from_numpy(x.view("int16")).to(device) for x in data["weights"]]
        ptrs = (C.c_void_p * len(Wd))(*[t.data_ptr() for t in Wd])
        a0 = torch.zeros(act.value // 2, dtype=torch.int16, device=device)
        a1 = torch.zeros(act.value // 2, dtype=torch.int16, device=device)
        out = torch.zeros(ob.value // 4, dtype=torch.float32, device=device)
        fn = lambda st: mgb.mgb_cnn_enqueue(st, arr, len(layers), _ptr(X), ptrs, _ptr(a0), _ptr(a1), _ptr(out), b, h, w)
        flops = sum(2.0 * b * L["h_out"] * L["w_out"] * L["c_out"] * 9 * L["c_in"] for L in layers)
        return Task(spec, dict(X=X, W=Wd, a0=a0, a1=a1, out=out, arr=arr, ptrs=ptrs), (mem.value, g, blk), fn,
                    "conv3x3_kernel", len(layers), alg_bytes=float(mem.value - act.value), alg_flops=flops,
                    wg_per_cu=int(mgb.mgb_cnn_residency(arr, len(layers), b, h, w)))
    raise ValueError(k)


MAX_WORKERS = 32      # the paper's pool for its largest (128-job) mix, Sec. V-E


def run_mix(sched, tasks, use_arrivals=True, time_scale=1.0, workers=None):
    """Push every task through probe -> (wait) -> launch -> sync -> complete with a pool of
    workers, each taking the next job in arrival order, running it to completion and pulling
    another (Sec. V-A).  The pool holds min(#tasks, 32) workers.

    With use_arrivals a job is not probed before t0 + arrival_i (it may additionally wait for a
    free worker; turnaround counts from its arrival either way); otherwise all probes are issued
    back to back in task-id order before anything runs (batch at t = 0) when the pool is as
    large as the mix, else as workers become free.
    Returns per-task records (times in seconds relative to t0) and the makespan."""
    n = len(tasks)
    n_workers = min(n, workers or MAX_WORKERS)
    rec = [dict(task_id=t.spec.task_id, kind=t.spec.kind) for t in tasks]
    errors = []
    placements = [None] * n
    order = sorted(range(n), key=lambda i: (tasks[i].spec.arrival_s, i)) if use_arrivals else list(range(n))
    cursor = [0]
    take = threading.Lock()
    torch.cuda.synchronize()
    t0 = time.perf_counter()

    pre_probed = (not use_arrivals) and n_workers >= n
    if pre_probed:
        for i, t in enumerate(tasks):
            rec[i]["arrival"] = 0.0
            rc, pl = sched.probe(t.spec.task_id, t.mem, t.grid, t.block, t.wg_per_cu)
            rec[i]["probe"] = time.perf_counter() - t0
            if rc != mgb.MGB_E_OOM:
                mgb.check(rc, "mgb_task_probe")
            placements[i] = (rc, pl)

    def crashed(i):
        # memory-blind packing (the CG baseline) let the job in where it could not fit: the job is
        # lost, which is the failure the paper's Sec. V-B counts
        rec[i]["crashed"] = True
        rec[i]["admit"] = rec[i]["done"] = time.perf_counter() - t0
        rec[i]["gpu_ms"] = 0.0
        rec[i]["granules"] = 0

    def run_one(i):
        t = tasks[i]
        if pre_probed:
            rc, pl = placements[i]
            if rc == mgb.MGB_E_OOM:
                return crashed(i)
        else:
            if use_arrivals:
                due = t0 + t.spec.arrival_s * time_scale
                while True:
                    dt = due - time.perf_counter()
                    if dt <= 0:
                        break
                    # (a sleep overshoots by 50-100 us: sleep short of the arrival, then yield in a loop)
                    time.sleep(dt - 2e-4 if dt > 4e-4 else 0)
                rec[i]["arrival"] = t.spec.arrival_s * time_scale
            else:
                rec[i]["arrival"] = 0.0
            rc, pl = sched.probe(t.spec.task_id, t.mem, t.grid, t.block, t.wg_per_cu)
            rec[i]["probe"] = time.perf_counter() - t0
            if rc == mgb.MGB_E_OOM:
                return crashed(i)
            mgb.check(rc, "mgb_task_probe")
        if rc == mgb.MGB_WAIT:
            rc, pl = sched.wait(pl.ticket)
            if rc == mgb.MGB_E_OOM:
                return crashed(i)
            mgb.check(rc, "mgb_task_wait")
        rec[i]["admit"] = time.perf_counter() - t0
        rec[i]["granules"] = pl.n_granules
        mgb.check(sched.launch(pl.ticket, t.enqueue), "mgb_task_launch")
        rc, ms = sched.sync(pl.ticket)
        mgb.check(rc, "mgb_task_sync")
        rec[i]["gpu_ms"] = ms
        rec[i]["done"] = time.perf_counter() - t0
        mgb.check(sched.complete(pl.ticket), "mgb_task_complete")

    def worker(w):
        try:
            if pre_probed:                     # one worker per job, job w
                run_one(w)
                return
            while True:
                with take:
                    if cursor[0] >= n:
                        return
                    i = order[cursor[0]]
                    cursor[0] += 1
                run_one(i)
        except Exception as e:   # noqa: BLE001
            errors.append((w, repr(e)))

    threads = [threading.Thread(target=worker, args=(w,)) for w in range(n_workers)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    torch.cuda.synchronize()
    makespan = time.perf_counter() - t0
    if errors:
        raise RuntimeError("mix failed: %r" % errors[:3])
    return rec, makespan


def summarize(rec, makespan):
    n_crashed = sum(1 for r in rec if r.get("crashed"))
    rec = [r for r in rec if not r.get("crashed")]       # only finished jobs count as throughput
    n = len(rec)
    if n == 0:
        return dict(tasks=0, crashed=n_crashed, tasks_per_s=0.0, mean_turnaround_ms=0.0, max_turnaround_ms=0.0,
                    makespan_ms=1e3 * makespan, mean_wait_ms=0.0)
    turn = [r["done"] - r["arrival"] for r in rec]
    last = max(r["done"] for r in rec)
    first = min(r["arrival"] for r in rec)
    return dict(tasks=n, crashed=n_crashed, tasks_per_s=n / (last - first), mean_turnaround_ms=1e3 * sum(turn) / n,
                max_turnaround_ms=1e3 * max(turn), makespan_ms=1e3 * makespan,
                mean_wait_ms=1e3 * sum(r["admit"] - r["probe"] for r in rec) / n)
