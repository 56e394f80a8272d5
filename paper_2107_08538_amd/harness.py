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
        self.kernel_name = kernel_name  # label of the task's kernels in reports: "jacobi" (the fused-sweep kernels of
                                        # jacobi.hip), "conv_net" (the layer launches of a net), "gemm_bf16_dma" (the
                                        # two DMA-ring kernels of gemm_bf16.hip), else the kernel itself
        self.launches = launches        # kernel launches per task (None if data dependent)
        self.alg_bytes = alg_bytes      # algorithmic HBM bytes of the whole task
        self.alg_flops = alg_flops
        self.edges = 0                  # stored (directed) edges of a graph task
        self.native = None              # (MGB_TASK_*, device pointers, dims, count, layers, weights) for mgb_pool_run


def build_task(spec, data, device="cuda:0"):
    """Upload one task's inputs (numpy arrays from the workload generators) and bind its entry points."""
    k, p = spec.kind, spec.params
    if k == "jacobi":
        n, it = p["n"], p["iters"]
        u0 = torch.from_numpy(data["u"]).to(device)
        u1 = u0.clone()
        probe = mgb.probe_of(mgb.mgb_jacobi_probe, n, it)
        fn = lambda st: mgb.mgb_jacobi_enqueue(st, _ptr(u0), _ptr(u1), n, it)
        t = Task(spec, dict(u0=u0, u1=u1), probe, fn, "jacobi", int(mgb.mgb_jacobi_launch_count(n, it)),
                 alg_bytes=8.0 * (n - 2) * (n - 2) * it, alg_flops=4.0 * (n - 2) * (n - 2) * it,
                 wg_per_cu=int(mgb.mgb_jacobi_residency(n)))
        t.native = (mgb.MGB_TASK_JACOBI, [u0, u1], [n, it], 0, None, None)
        return t
    if k == "gemm_f32":
        m, n, kk = p["m"], p["n"], p["k"]
        A, B = torch.from_numpy(data["a"]).to(device), torch.from_numpy(data["b"]).to(device)
        Cc = torch.zeros(m, n, device=device)
        probe = mgb.probe_of(mgb.mgb_gemm_f32_probe, m, n, kk)
        fn = lambda st: mgb.mgb_gemm_f32_enqueue(st, _ptr(A), _ptr(B), _ptr(Cc), m, n, kk)
        t = Task(spec, dict(A=A, B=B, C=Cc), probe, fn, "gemm_f32_dma_kernel", 1,
                 alg_bytes=4.0 * (m * kk + kk * n + m * n), alg_flops=2.0 * m * n * kk,
                 wg_per_cu=int(mgb.mgb_gemm_f32_residency(m, n, kk)))
        t.native = (mgb.MGB_TASK_GEMM_F32, [A, B, Cc], [m, n, kk], 0, None, None)
        return t
    if k == "gemm_bf16":
        m, n, kk = p["m"], p["n"], p["k"]
        A = torch.from_numpy(data["a"].view("int16")).to(device)
        B = torch.from_numpy(data["b"].view("int16")).to(device)
        Cc = torch.zeros(m, n, device=device)
        probe = mgb.probe_of(mgb.mgb_gemm_bf16_probe, m, n, kk)
        fn = lambda st: mgb.mgb_gemm_bf16_enqueue(st, _ptr(A), _ptr(B), _ptr(Cc), m, n, kk)
        t = Task(spec, dict(A=A, B=B, C=Cc), probe, fn, "gemm_bf16_dma", 1,
                 alg_bytes=2.0 * (m * kk + kk * n) + 4.0 * m * n, alg_flops=2.0 * m * n * kk,
                 wg_per_cu=int(mgb.mgb_gemm_bf16_residency(m, n, kk)))
        t.native = (mgb.MGB_TASK_GEMM_BF16, [A, B, Cc], [m, n, kk], 0, None, None)
        return t
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
        t.native = (mgb.MGB_TASK_BFS, [rp, ci, level, work], [n, 0], m_edges, None, None)
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
        t = Task(spec, dict(X=X, W=Wd, a0=a0, a1=a1, out=out, arr=arr, ptrs=ptrs), (mem.value, g, blk), fn,
                 "conv_net", len(layers), alg_bytes=float(mem.value - act.value), alg_flops=flops,
                 wg_per_cu=int(mgb.mgb_cnn_residency(arr, len(layers), b, h, w)))
        t.native = (mgb.MGB_TASK_CNN, [X, a0, a1, out], [b, h, w], len(layers), arr, ptrs)
        return t
    raise ValueError(k)


MAX_WORKERS = 32      # the paper's pool for its largest (128-job) mix, Sec. V-E


def run_mix(sched, tasks, use_arrivals=True, time_scale=1.0, workers=None, release_on_stream=False):
    """Push every task through probe -> (wait) -> launch -> sync -> complete with a pool of
    workers, each taking the next job in arrival order, running it to completion and pulling
    another (Sec. V-A).  The pool holds min(#tasks, 32) workers.  With release_on_stream a task
    hands its resources back as soon as its kernels are enqueued (mgb_task_complete_on_stream) and
    only then waits for them.

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
    t0_ns = time.monotonic_ns()

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
        rec[i]["ticket"] = pl.ticket
        mgb.check(sched.launch(pl.ticket, t.enqueue), "mgb_task_launch")
        if release_on_stream:
            mgb.check(sched.complete_on_stream(pl.ticket), "mgb_task_complete_on_stream")
        rc, ms = sched.sync(pl.ticket)
        mgb.check(rc, "mgb_task_sync")
        rec[i]["gpu_ms"] = ms
        rec[i]["done"] = time.perf_counter() - t0
        if not release_on_stream:
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
    # what the scheduler itself recorded of every task (probe, admission, release, end of its
    # kernels): the figures of summarize() are computed by the library from these
    tickets = [r["ticket"] for r in rec if "ticket" in r]
    by_ticket = {}
    if tickets:
        lo, hi = min(tickets), max(tickets)
        got, n_got = sched.records(lo, hi - lo + 1)
        by_ticket = {got[j].ticket: got[j] for j in range(n_got)}
    for i, r in enumerate(rec):
        r["arrival_ns"] = t0_ns + int(1e9 * r["arrival"])
        r["record"] = by_ticket.get(r.get("ticket"))
    return rec, makespan


def run_mix_native(sched, tasks, use_arrivals=True, time_scale=1.0, workers=None, release_on_stream=False):
    """run_mix with the worker pool inside the library (mgb_pool_run): the same jobs, the same
    order of calls per job, native threads.  Returns the same per-task records."""
    n = len(tasks)
    descs = (mgb.mgb_task_desc * n)()
    for i, t in enumerate(tasks):
        kind, ptrs, dims, count, layers, weights = t.native
        d = descs[i]
        d.kind, d.task_id, d.count = kind, t.spec.task_id, count
        d.arrival_ns = int(1e9 * t.spec.arrival_s * time_scale) if use_arrivals else 0
        for j, x in enumerate(ptrs):
            d.ptr[j] = x.data_ptr()
        for j, x in enumerate(dims):
            d.dim[j] = x
        if layers is not None:
            d.layers = C.cast(layers, C.POINTER(mgb.mgb_conv_layer))
            d.weights = C.cast(weights, C.POINTER(C.c_void_p))
    res = (mgb.mgb_pool_result * n)()
    start = C.c_uint64(0)
    flags = (mgb.MGB_POOL_ARRIVALS if use_arrivals else 0) | (mgb.MGB_POOL_RELEASE_ON_STREAM if release_on_stream else 0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    mgb.check(mgb.mgb_pool_run(sched.h, descs, n, min(n, workers or MAX_WORKERS), flags, res, C.byref(start)), "mgb_pool_run")
    torch.cuda.synchronize()
    makespan = time.perf_counter() - t0
    rec = []
    for i, t in enumerate(tasks):
        r, a = res[i], res[i].record
        row = dict(task_id=t.spec.task_id, kind=t.spec.kind, arrival_ns=int(r.arrival_ns),
                   arrival=1e-9 * (r.arrival_ns - start.value), ticket=int(r.ticket))
        if r.status == mgb.MGB_E_OOM:
            row.update(crashed=True, gpu_ms=0.0, granules=0, record=None)
        else:
            mgb.check(r.status, "job %d in mgb_pool_run" % t.spec.task_id)
            rcopy = mgb.mgb_task_record.from_buffer_copy(a)
            row.update(probe=1e-9 * (a.probe_ns - start.value), admit=1e-9 * (a.admit_ns - start.value),
                       done=1e-9 * (a.done_ns - start.value), gpu_ms=a.gpu_ms, granules=int(a.demand), record=rcopy)
            if t.spec.kind == "bfs":
                t.depth.value = r.aux
        rec.append(row)
    return rec, makespan


def summarize(rec, makespan, ref_gpu_ms=None):
    """Throughput, turnaround, waiting time (Sec. V-A) and, given each task's time on a dedicated
    device, kernel slowdown (Sec. V, last table) of one pass: mgb_accounting on the scheduler's own
    task records; this function only marshals and formats."""
    n = len(rec)
    recs = (mgb.mgb_task_record * n)()
    arr = (C.c_uint64 * n)()
    ref = (C.c_double * n)()
    for i, r in enumerate(rec):
        if r.get("crashed") or r.get("record") is None:
            recs[i].status = mgb.MGB_E_OOM if r.get("crashed") else mgb.MGB_WAIT
        else:
            recs[i] = r["record"]
        arr[i] = r["arrival_ns"]
        ref[i] = ref_gpu_ms[i] if ref_gpu_ms is not None else 0.0
    out = mgb.mgb_summary()
    mgb.check(mgb.mgb_accounting(recs, n, arr, ref, C.byref(out)), "mgb_accounting")
    return dict(tasks=int(out.n_done), crashed=int(out.n_crashed), tasks_per_s=out.tasks_per_s,
                mean_turnaround_ms=out.mean_turnaround_ms, max_turnaround_ms=out.max_turnaround_ms,
                makespan_ms=out.makespan_ms, mean_wait_ms=out.mean_wait_ms, max_wait_ms=out.max_wait_ms,
                gpu_busy_ms=out.gpu_busy_ms, max_slowdown=out.max_slowdown, mean_slowdown=out.mean_slowdown,
                host_makespan_ms=1e3 * makespan)
