#!/usr/bin/env python3
"""Bench: one "step" = one pass of a whole task mix (default Mix-16: 16 tasks, Poisson arrivals,
Jacobi 4096^2 x100 / fp32 GEMM 4096^3 / BFS 2^20) through probe -> admit -> CU partition ->
launch -> complete on one MI355X, inputs resident in HBM.  Prints ONE JSON line."""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--mix", default="mix16", choices=["mix4", "mix16", "cnn8", "mixed128", "kinds5"])
    ap.add_argument("--policy", default="hard", choices=["hard", "soft", "serial"])
    ap.add_argument("--queue", default="backfill", choices=["backfill", "fifo"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip serialised / alone / batch comparisons")
    ap.add_argument("--seed", type=int, default=None)
    return ap.parse_args()


# HBM-side bytes per launch from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs summarised in
# profiles/mix16_hbm_traffic.md (each counter scaled by its reading for the 1 GiB stream copy).
# Valid for the kernels as they stand in csrc/ and for the Mix-16 task shapes only.
MEASURED_TRAFFIC_BYTES = {
    ("mix16", "gemm_f32_dma_kernel"): 470.4e6,  # per 4096^3 launch
    ("mix16", "jacobi_stream"): 182.1e6,       # per launch (2 eight-sweep + 12 seven-sweep launches per task)
    ("mix16", "bfs_level"): 20.7e6,            # per level launch, averaged over the 8 launches of a traversal
}


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def cpu_baseline(spec):
    """Serial CPU checker timed on a bounded sample of the same workload, scaled by work."""
    import numpy as np
    import oracle
    import workloads as W
    per_kind, sample = {}, []
    kinds = {}
    for t in spec["tasks"]:
        kinds.setdefault((t.kind, tuple(sorted(t.params.items()))), t)
    for (kind, _), t in kinds.items():
        p = t.params
        if kind == "jacobi":
            it = max(1, min(p["iters"], int(3e8 // (p["n"] * p["n"]))))
            u = W.jacobi_field(1, p["n"])
            t0 = time.perf_counter(); oracle.jacobi_f32(u, it); dt = time.perf_counter() - t0
            per_kind[(kind, tuple(sorted(p.items())))] = dt * p["iters"] / it
            sample.append("jacobi %d^2 x%d of %d sweeps" % (p["n"], it, p["iters"]))
        elif kind in ("gemm_f32", "gemm_bf16"):
            s = min(p["m"], 1024)
            a, b = W.gemm_operands_f32(1, s, s, s)
            t0 = time.perf_counter(); oracle.gemm_f32(a, b); dt = time.perf_counter() - t0
            per_kind[(kind, tuple(sorted(p.items())))] = dt * (p["m"] * p["n"] * p["k"]) / float(s) ** 3
            sample.append("gemm %d^3 scaled by flops to %dx%dx%d (extrapolated)" % (s, p["m"], p["n"], p["k"]))
        elif kind == "bfs":
            n = min(p["n"], 1 << 20)
            rp, ci = W.er_graph_csr(1, n, p["degree"])
            t0 = time.perf_counter(); oracle.bfs(rp, ci, 0); dt = time.perf_counter() - t0
            per_kind[(kind, tuple(sorted(p.items())))] = dt * p["n"] / n
            sample.append("bfs n=%d degree %d" % (n, p["degree"]))
        elif kind == "cnn":
            h = 52
            layers = W.cnn_layers(h, h)
            wts = W.cnn_weights(1, layers)
            x = W.cnn_input(1, 1, h, h)
            t0 = time.perf_counter(); oracle.cnn_forward(x, wts, [L["stride"] for L in layers]); dt = time.perf_counter() - t0
            per_kind[(kind, tuple(sorted(p.items())))] = dt * p["batch"] * (p["h"] * p["w"]) / float(h * h)
            sample.append("cnn %dx%d batch 1 scaled by pixels (extrapolated)" % (h, h))
    total = sum(per_kind[(t.kind, tuple(sorted(t.params.items())))] for t in spec["tasks"])
    # serial FIFO on one core: task i starts when it has arrived and the previous one is done
    clock, turn = 0.0, []
    for t in spec["tasks"]:
        clock = max(clock, t.arrival_s) + per_kind[(t.kind, tuple(sorted(t.params.items())))]
        turn.append(clock - t.arrival_s)
    model = ""
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return dict(value=len(spec["tasks"]) / clock, unit="tasks/s", cores=1, kind="oracle",
                sample="; ".join(sample), est_seconds_per_mix=total,
                mean_turnaround_ms=1e3 * sum(turn) / len(turn), nproc=os.cpu_count(), cpu_model=model)


def lazy_leg(mgb, cap):
    """One fp32 GEMM 1024^3 task built through the lazy runtime (Sec. III-A): host time of each
    stage.  Host buffers cross PCIe here, unlike the timed region of the bench."""
    import ctypes as C
    import numpy as np
    import workloads as W
    n = 1024
    a, b = W.gemm_operands_f32(1, n, n, n)
    out = np.empty((n, n), np.float32)
    s = mgb.Sched(mem_cap_bytes=cap)
    z = mgb.Lazy(s)
    mem, grid, block = mgb.probe_of(mgb.mgb_gemm_f32_probe, n, n, n)
    stages = dict(record_ms=0.0, prepare_ms=0.0, kernel_and_copy_back_ms=0.0, free_ms=0.0)
    reps = 5
    for rep in range(reps + 1):
        t0 = time.perf_counter()
        pa, pb, pc = (z.malloc(n * n * 4)[1] for _ in range(3))
        z.memcpy_h2d(pa, a.ctypes.data, a.nbytes)
        z.memcpy_h2d(pb, b.ctypes.data, b.nbytes)
        t1 = time.perf_counter()
        rc, real, pl = z.launch_prepare(rep, [pa, pb, pc], grid, block)
        mgb.check(rc, "mgb_lazy_launch_prepare")
        t2 = time.perf_counter()
        mgb.check(mgb.mgb_gemm_f32_enqueue(pl.stream, real[0], real[1], real[2], n, n, n), "mgb_gemm_f32_enqueue")
        mgb.check(z.memcpy_d2h(out.ctypes.data, pc, out.nbytes), "mgb_lazy_memcpy_d2h")
        t3 = time.perf_counter()
        for p in (pa, pb, pc):
            mgb.check(z.free(p), "mgb_lazy_free")
        t4 = time.perf_counter()
        if rep:                                   # the first pass warms the allocator
            for k, dt in zip(stages, (t1 - t0, t2 - t1, t3 - t2, t4 - t3)):
                stages[k] += 1e3 * dt / reps
    z.destroy()
    s.destroy()
    return dict(task="gemm_f32 1024^3, 12 MiB footprint discovered at the launch", footprint_bytes=mem,
                **{k: round(v, 3) for k, v in stages.items()})


def ipc_leg(mgb):
    """Cost of reaching the scheduler through the shared-memory front end (Sec. IV): probe +
    complete of a small task, through a client connection and directly.  Decisions only (null
    backend), the client sits in this process; a client in another process pays the same two
    semaphore hand-offs per call."""
    s = mgb.Sched(backend=mgb.MGB_BACKEND_NULL)
    sv = mgb.Server(s, "bench%d" % os.getpid(), 2)
    c = mgb.Client("bench%d" % os.getpid())
    n = 2000

    def loop(obj):
        t0 = time.perf_counter()
        for i in range(n):
            rc, pl = obj.probe(i, 1 << 20, (64, 1, 1), (256, 1, 1))
            obj.complete(pl.ticket)
        return 1e6 * (time.perf_counter() - t0) / n
    loop(c)
    via, direct = loop(c), loop(s)
    c.disconnect()
    sv.stop()
    s.destroy()
    return dict(probe_plus_complete_us=round(via, 2), in_process_us=round(direct, 2))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures the one-GPU co-execution path only: run with --gpus 1 "
              "(tasks never communicate; more GPUs would be more independent schedulers)", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("no GPU visible: the HIP path cannot run and there is no CPU fallback", file=sys.stderr)
        sys.exit(3)
    if not os.path.exists(os.path.join(ROOT, "paper_2107_08538_amd", "libmgb.so")):
        import __graft_entry__
        __graft_entry__.build()
    import paper_2107_08538_amd as mgb
    from paper_2107_08538_amd import harness
    import workloads as W

    mixfn = W.MIXES[args.mix]
    spec = mixfn(args.seed) if args.seed is not None else mixfn()
    t_gen = time.perf_counter()
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:   # numpy releases the GIL
        data = list(ex.map(W.task_data, spec["tasks"]))
    tasks = [harness.build_task(t, d) for t, d in zip(spec["tasks"], data)]
    del data
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen

    # measured stream-copy ceiling (plain copy kernel of known size, also the counter calibration point)
    import ctypes as C
    cbytes = 1 << 30
    csrc = torch.empty(cbytes, dtype=torch.uint8, device="cuda:0")
    cdst = torch.empty(cbytes, dtype=torch.uint8, device="cuda:0")
    cs = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    mgb.mgb_copy_enqueue(cs, C.c_void_p(cdst.data_ptr()), C.c_void_p(csrc.data_ptr()), cbytes)
    e0.record()
    for _ in range(5):
        mgb.mgb_copy_enqueue(cs, C.c_void_p(cdst.data_ptr()), C.c_void_p(csrc.data_ptr()), cbytes)
    e1.record()
    torch.cuda.synchronize()
    copy_gbps = 5 * 2 * cbytes / (e0.elapsed_time(e1) / 1e3) / 1e9
    del csrc, cdst
    # measured matrix-core ceilings: MFMA instructions on registers only, one wave per SIMD on every CU
    mfma_tflops = {}
    mout = torch.empty(1024 * 256, dtype=torch.float32, device="cuda:0")
    for name, is_bf16 in (("f32", 0), ("bf16", 1)):
        fl = C.c_double(0.0)
        mgb.check(mgb.mgb_mfma_loop_enqueue(cs, is_bf16, 1024, 4096, C.c_void_p(mout.data_ptr()), C.byref(fl)),
                  "mgb_mfma_loop_enqueue")
        e0.record()
        for _ in range(3):
            mgb.mgb_mfma_loop_enqueue(cs, is_bf16, 1024, 4096, C.c_void_p(mout.data_ptr()), C.byref(fl))
        e1.record()
        torch.cuda.synchronize()
        mfma_tflops[name] = 3 * fl.value / (e0.elapsed_time(e1) / 1e3) / 1e12
    del mout

    pol = dict(hard=mgb.MGB_POLICY_HARD, soft=mgb.MGB_POLICY_SOFT, serial=mgb.MGB_POLICY_SERIAL)[args.policy]
    qm = dict(backfill=mgb.MGB_QUEUE_BACKFILL, fifo=mgb.MGB_QUEUE_FIFO)[args.queue]
    free_b, total_b = torch.cuda.mem_get_info()
    cap = min(spec["cap_bytes"], total_b)
    sched = mgb.Sched(policy=pol, queue_mode=qm, mem_cap_bytes=cap)

    log("inputs resident (%d tasks, %.1f s); stream copy %.0f GB/s; MFMA loop %.0f (f32) / %.0f (bf16) TFLOP/s"
        % (len(tasks), t_gen, copy_gbps, mfma_tflops["f32"], mfma_tflops["bf16"]))
    for _ in range(args.warmup):
        harness.run_mix(sched, tasks)
    log("warm-up done, %d masked streams" % sched.stats().n_streams)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    runs = []
    for _ in range(args.steps):
        runs.append(harness.run_mix(sched, tasks))
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    n_tasks = len(tasks)
    log("timed region done: %d steps in %.3f s, %d masked streams" % (args.steps, elapsed, sched.stats().n_streams))
    sums = [harness.summarize(r, m) for r, m in runs]
    value = n_tasks * args.steps / elapsed
    mean_turn = sum(s["mean_turnaround_ms"] for s in sums) / len(sums)

    # per-kernel figures from the timed region (HIP events bracket each task on its own stream)
    kern = {}
    for rec, _ in runs:
        for r, t in zip(rec, tasks):
            k = kern.setdefault(t.kernel_name, dict(ms=0.0, launches=0, tasks=0, bytes=0.0, flops=0.0, edges=0))
            launches = t.launches if t.launches is not None else max(1, int(t.depth.value))
            k["ms"] += r["gpu_ms"]; k["launches"] += launches; k["tasks"] += 1
            k["bytes"] += t.alg_bytes; k["flops"] += t.alg_flops; k["edges"] += t.edges
    dominant = max(kern, key=lambda n: kern[n]["ms"])
    kd = kern[dominant]
    peaks = dict(jacobi_sweeps=("hbm", 8000.0, "GB/s"), jacobi_stream=("hbm", 8000.0, "GB/s"), bfs_level=("hbm", 8000.0, "GB/s"),
                 gemm_f32_dma_kernel=("mfma", 157.3, "TFLOP/s"), gemm_bf16_dma_kernel=("mfma", 2500.0, "TFLOP/s"),
                 conv3x3_kernel=("mfma", 2500.0, "TFLOP/s"))

    def measured_ceiling(name):
        # what this device sustains on the same resource with nothing else in the way: the plain copy
        # kernel for HBM-bound kernels, the register-only MFMA loop of the kernel's dtype otherwise
        if peaks[name][0] == "hbm":
            return copy_gbps
        return mfma_tflops["f32" if name == "gemm_f32_dma_kernel" else "bf16"]

    def roof(name, k):
        bound, peak, unit = peaks[name]
        work = k["bytes"] / 1e9 if bound == "hbm" else k["flops"] / 1e12
        ach = work / (k["ms"] / 1e3)
        out = dict(kernel=name, bound=bound, achieved=round(ach, 2), peak=peak, unit=unit,
                   frac=round(ach / peak, 4), measured_ceiling=round(measured_ceiling(name), 1),
                   frac_of_measured=round(ach / measured_ceiling(name), 4), traffic=MEASURED_TRAFFIC_BYTES.get((args.mix, name)),
                   avg_launch_us=round(1e3 * k["ms"] / k["launches"], 2), launches=k["launches"])
        if k["edges"]:
            out["gteps"] = round(k["edges"] / (k["ms"] / 1e3) / 1e9, 2)      # stored directed edges per second of traversal
        return out

    out = dict(metric="aggregate tasks/s through probe+admit+partition+launch+complete (with mean turnaround, max slowdown)",
               value=round(value, 2), unit="tasks/s", n_gpus=1, steps=args.steps, warmup=args.warmup,
               ms_per_step=round(1e3 * elapsed / args.steps, 3), higher_is_better=True, scaling="weak",
               vs_baseline=None, dtype="f32", data="synthetic",
               config=dict(workload="%s: %s" % (spec["name"], ", ".join(sorted({t.kind for t in spec["tasks"]}))),
                           policy=args.policy, queue=args.queue, tasks=n_tasks, workers=min(n_tasks, harness.MAX_WORKERS),
                           cap_bytes=cap, granule_cus=int(sched.desc.granule_cus), n_cu=256),
               mean_turnaround_ms=round(mean_turn, 3),
               mean_wait_ms=round(sum(s["mean_wait_ms"] for s in sums) / len(sums), 3),
               input_gen_s=round(t_gen, 1), stream_copy_gbps=round(copy_gbps, 1),
               mfma_loop_tflops={k: round(v, 1) for k, v in mfma_tflops.items()})
    out["roofline"] = roof(dominant, kd)
    out["kernels"] = [roof(n, k) for n, k in kern.items() if n != dominant]

    if not args.no_extras:
        # the same mix, serialised: one task at a time on all 256 CUs in arrival order
        log("serialised comparator")
        ser = mgb.Sched(policy=mgb.MGB_POLICY_SERIAL, queue_mode=mgb.MGB_QUEUE_FIFO, mem_cap_bytes=cap)
        harness.run_mix(ser, tasks)
        t1 = time.perf_counter()
        sruns = [harness.run_mix(ser, tasks) for _ in range(max(2, args.steps // 2))]
        torch.cuda.synchronize()
        sel = time.perf_counter() - t1
        ssum = [harness.summarize(r, m) for r, m in sruns]
        out["serialised_gpu"] = dict(tasks_per_s=round(n_tasks * len(sruns) / sel, 2),
                                     mean_turnaround_ms=round(sum(s["mean_turnaround_ms"] for s in ssum) / len(ssum), 3))
        # kernel slowdown as the paper defines it (Sec. V, last experiment): GPU time of a task in the
        # shared run against the same task in the single-assignment run of the same workload
        # (per task the median over the passes: one pass in which a 0.2 ms task meets a host hiccup
        # would otherwise decide the maximum over tasks)
        def mid(v):
            v = sorted(v)
            return 0.5 * (v[(len(v) - 1) // 2] + v[len(v) // 2])
        co = [mid([run[0][i]["gpu_ms"] for run in runs]) for i in range(n_tasks)]
        sa = [mid([run[0][i]["gpu_ms"] for run in sruns]) for i in range(n_tasks)]
        slow = [c / a - 1.0 for c, a in zip(co, sa)]
        kinds = sorted({t.spec.kind for t in tasks})
        out["max_slowdown_pct"] = round(100 * max(slow), 2)
        out["mean_slowdown_pct"] = round(100 * sum(slow) / len(slow), 2)
        out["slowdown_by_kind_pct"] = {k: round(100 * max(s for s, t in zip(slow, tasks) if t.spec.kind == k), 2)
                                       for k in kinds}
        out["corun_gpu_ms"] = {k: round(max(c for c, t in zip(co, tasks) if t.spec.kind == k), 4) for k in kinds}
        out["serialised_gpu_ms"] = {k: round(max(c for c, t in zip(sa, tasks) if t.spec.kind == k), 4) for k in kinds}
        # each task alone, back to back on a busy (clocked-up) device: the kernels' own speed
        log("tasks alone")
        alone = []
        for t in tasks:
            harness.run_mix(ser, [t], use_arrivals=False)
            vals = [harness.run_mix(ser, [t], use_arrivals=False)[0][0]["gpu_ms"] for _ in range(4)]
            alone.append(sum(vals) / len(vals))
        out["alone_back_to_back_gpu_ms"] = {k: round(min(a for a, t in zip(alone, tasks) if t.spec.kind == k), 4)
                                            for k in kinds}
        # the dominant kernel's own speed: the same figure as `roofline`, from the back-to-back launches
        # (the timed region above has idle gaps between arrivals, and the clocks ramp after each)
        da = [(a, t) for a, t in zip(alone, tasks) if t.kernel_name == dominant]
        if da:
            bound, peak, unit = peaks[dominant]
            work = sum((t.alg_bytes / 1e9 if bound == "hbm" else t.alg_flops / 1e12) for _, t in da)
            ach = work / (sum(a for a, _ in da) / 1e3)
            out["roofline_back_to_back"] = dict(kernel=dominant, bound=bound, achieved=round(ach, 2), peak=peak,
                                                unit=unit, frac=round(ach / peak, 4),
                                                frac_of_measured=round(ach / measured_ceiling(dominant), 4))
        out["speedup_vs_serialised"] = dict(
            throughput=round(value / out["serialised_gpu"]["tasks_per_s"], 4),
            turnaround=round(out["serialised_gpu"]["mean_turnaround_ms"] / mean_turn, 4))
        # batch variant (all tasks queued at t = 0, the paper's setting): capacity rather than arrival bound
        log("batch at t=0")
        # (medians of five passes: the worker threads' scheduling makes single passes vary by several per cent)
        def med(runs, key):
            return sorted(x[key] for x in runs)[len(runs) // 2]
        harness.run_mix(sched, tasks, use_arrivals=False)
        b = [harness.summarize(*harness.run_mix(sched, tasks, use_arrivals=False)) for _ in range(5)]
        bs = [harness.summarize(*harness.run_mix(ser, tasks, use_arrivals=False)) for _ in range(5)]
        out["batch_t0"] = dict(tasks_per_s=round(med(b, "tasks_per_s"), 2),
                               mean_turnaround_ms=round(med(b, "mean_turnaround_ms"), 3),
                               tasks_per_s_min_max=[round(min(x["tasks_per_s"] for x in b), 1), round(max(x["tasks_per_s"] for x in b), 1)],
                               serialised_tasks_per_s=round(med(bs, "tasks_per_s"), 2),
                               serialised_mean_turnaround_ms=round(med(bs, "mean_turnaround_ms"), 3))
        # what the co-run sustains as a whole: the tasks' algorithmic HBM bytes and flops over the makespan
        mk = 1e-3 * med(b, "makespan_ms")
        out["batch_t0"]["corun_algorithmic_hbm_gbs"] = round(sum(t.alg_bytes for t in tasks) / mk / 1e9, 1)
        out["batch_t0"]["corun_tflops"] = round(sum(t.alg_flops for t in tasks) / mk / 1e12, 2)
        # the other policies on the same mix: Alg. 3 analogue (overlapping masks), FIFO queue,
        # HARD with one workgroup per CU as the residency limit ("spread": a task gets as many
        # CUs as it has workgroups, so only tasks that cannot fill the device share it), and the
        # memory-blind CG baseline of Sec. IV at four jobs per device
        sched.destroy()
        sched = None
        sweep = {}
        for name, pol2, q2, wgcu, ratio in (("soft_backfill", mgb.MGB_POLICY_SOFT, mgb.MGB_QUEUE_BACKFILL, 32, 8),
                                            ("hard_fifo", mgb.MGB_POLICY_HARD, mgb.MGB_QUEUE_FIFO, 32, 8),
                                            ("hard_spread", mgb.MGB_POLICY_HARD, mgb.MGB_QUEUE_BACKFILL, 1, 8),
                                            ("cg_ratio4", mgb.MGB_POLICY_CG, mgb.MGB_QUEUE_BACKFILL, 32, 4)):
            log("policy sweep: " + name)
            s2 = mgb.Sched(policy=pol2, queue_mode=q2, mem_cap_bytes=cap, max_wg_per_cu=wgcu, max_running=ratio)
            harness.run_mix(s2, tasks)
            a = [harness.summarize(*harness.run_mix(s2, tasks)) for _ in range(3)]
            harness.run_mix(s2, tasks, use_arrivals=False)
            bb = [harness.summarize(*harness.run_mix(s2, tasks, use_arrivals=False)) for _ in range(5)]
            sweep[name] = dict(tasks_per_s=round(sum(x["tasks_per_s"] for x in a) / 3, 2),
                               mean_turnaround_ms=round(sum(x["mean_turnaround_ms"] for x in a) / 3, 3),
                               batch_tasks_per_s=round(med(bb, "tasks_per_s"), 2),
                               batch_mean_turnaround_ms=round(med(bb, "mean_turnaround_ms"), 3))
            s2.destroy()
        out["other_policies"] = sweep
        ser.destroy()
        log("lazy runtime")
        out["lazy_runtime"] = lazy_leg(mgb, cap)
        log("multi-process front end")
        out["ipc_front_end"] = ipc_leg(mgb)
    if not args.no_cpu_baseline:
        log("cpu baseline")
        out["cpu_baseline"] = cpu_baseline(spec)
    if sched is not None:
        sched.destroy()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
