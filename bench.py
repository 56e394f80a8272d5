#!/usr/bin/env python3
"""Bench: one "step" = one pass of a whole task mix (default Mix-16: 16 tasks, Poisson arrivals,
Jacobi 4096^2 x100 / fp32 GEMM 4096^3 / BFS 2^20) through probe -> admit -> CU partition ->
launch -> release on one MI355X, inputs resident in HBM.  Prints ONE JSON line."""
import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--mix", default="mix16", choices=["mix4", "mix16", "cnn8", "mixed128", "kinds5"])
    ap.add_argument("--policy", default="hard", choices=["hard", "soft", "serial"])
    ap.add_argument("--queue", default="backfill", choices=["backfill", "fifo"])
    ap.add_argument("--harness", default="native", choices=["native", "python"],
                    help="worker pool inside the library (mgb_pool_run) or Python threads over the same calls")
    ap.add_argument("--release", default="stream", choices=["stream", "host"],
                    help="hand resources back when the last kernel is enqueued (ordered on the device) or when the host has seen it finish")
    ap.add_argument("--batch", action="store_true", help="timed region with all tasks queued at t = 0 instead of arrivals")
    ap.add_argument("--workers", type=int, default=None, help="size of the worker pool (default: min(#tasks, 32), the paper's largest pool)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip serialised / alone / batch comparisons")
    ap.add_argument("--no-other-mixes", action="store_true", help="skip the batch legs of CNN-8, Mixed-128 and the memory-tight mix")
    ap.add_argument("--vendor-libraries", action="store_true",
                    help="also time the same GEMMs and the conv chain through the vendor libraries torch calls "
                         "(rocBLAS / hipBLASLt, MIOpen) on this box and report them beside this library's kernels")
    ap.add_argument("--dump-records", default=None, help="write the last timed pass's task records (JSON) to this path")
    ap.add_argument("--seed", type=int, default=None)
    return ap.parse_args()


TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "mix16_hbm_traffic.md")


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def med(v):
    v = sorted(v)
    return 0.5 * (v[(len(v) - 1) // 2] + v[len(v) // 2])


def cpu_baseline(spec):
    """Serial CPU checker timed on a bounded sample of the same workload, scaled by work."""
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


def other_mixes(mgb, harness, W, run, total_b, on_stream):
    """The mixes in which tasks do share the device, all jobs queued at t = 0 (the paper's setting), HARD
    against single assignment through the same pool; and the memory-tight mix on which packing by a
    fixed jobs-per-device ratio without looking at footprints (Sec. IV's CG baseline) loses jobs."""
    import torch
    from concurrent.futures import ThreadPoolExecutor
    res = {}
    for name, passes in (("cnn8", 7), ("mixed128", 3)):
        log("other mixes: " + name)
        spec = W.MIXES[name]()
        with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
            data = list(ex.map(W.task_data, spec["tasks"]))
        tasks = [harness.build_task(t, d) for t, d in zip(spec["tasks"], data)]
        del data
        cap = min(spec["cap_bytes"], total_b)
        row = {}
        for key, pol, q, ros in (("hard", mgb.MGB_POLICY_HARD, mgb.MGB_QUEUE_BACKFILL, on_stream),
                                 ("serialised", mgb.MGB_POLICY_SERIAL, mgb.MGB_QUEUE_FIFO, False)):
            s = mgb.Sched(policy=pol, queue_mode=q, mem_cap_bytes=cap)
            run(s, tasks, use_arrivals=False, release_on_stream=ros)
            ss = [harness.summarize(*run(s, tasks, use_arrivals=False, release_on_stream=ros)) for _ in range(passes)]
            row[key] = dict(tasks_per_s=round(med([x["tasks_per_s"] for x in ss]), 1),
                            mean_turnaround_ms=round(med([x["mean_turnaround_ms"] for x in ss]), 3),
                            mean_wait_ms=round(med([x["mean_wait_ms"] for x in ss]), 3))
            s.destroy()
        row["throughput_vs_serialised"] = round(row["hard"]["tasks_per_s"] / row["serialised"]["tasks_per_s"], 4)
        row["turnaround_vs_serialised"] = round(row["serialised"]["mean_turnaround_ms"] / row["hard"]["mean_turnaround_ms"], 4)
        row["tasks"] = len(tasks)
        res[name + "_batch_t0"] = row
        del tasks
        torch.cuda.empty_cache()
    log("other mixes: memory-tight")
    spec = W.pressure32(seed=9, scale=1 / 32)                     # 32 tasks whose footprints sum to 1.5 x the cap
    tasks = [harness.build_task(t, W.task_data(t)) for t in spec["tasks"]]
    row = {}
    for key, pol, ratio in (("hard", mgb.MGB_POLICY_HARD, 8), ("cg_ratio8", mgb.MGB_POLICY_CG, 8), ("cg_ratio32", mgb.MGB_POLICY_CG, 32)):
        s = mgb.Sched(policy=pol, max_running=ratio, mem_cap_bytes=spec["cap_bytes"])
        sm = harness.summarize(*run(s, tasks, use_arrivals=False))
        row[key] = dict(finished=sm["tasks"], lost_to_out_of_memory=sm["crashed"])
        s.destroy()
    res["memory_tight_32_tasks"] = row
    return res


# what bounds each kernel, its peak and the unit of `achieved`.  The Jacobi kernels fuse up to eight
# sweeps per pass over the grid, so they are not bound by 8 bytes per update through HBM but by
# plain fp32 vector arithmetic: adds and one multiply per update, no fused multiply-adds, no packed
# fp32 (not used in this code base), i.e. one flop per lane per issue slot.  That rate is
# 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz = 39.3 Tflop/s (the published 157.3 TFLOP/s counts a
# packed fused multiply-add as four flops per lane and clock).
VALU_PLAIN_TFLOPS = 256 * 4 * 16 * 2.4e9 / 1e12
PEAKS = dict(jacobi=("alu", VALU_PLAIN_TFLOPS, "TFLOP/s"), bfs_level=("hbm", 8000.0, "GB/s"),
             gemm_f32_dma_kernel=("mfma", 157.3, "TFLOP/s"), gemm_bf16_dma=("mfma", 2500.0, "TFLOP/s"),
             conv_net=("mfma", 2500.0, "TFLOP/s"))


def vendor_libraries(torch, mgb, W, log):
    """The task kernels against the vendor libraries on the same box and the same shapes, back to back on
    one stream: fp32 and bf16 GEMM through torch.matmul (rocBLAS / hipBLASLt), the ten-layer conv chain through
    torch's conv2d + relu per layer (MIOpen, channels-last bf16).  Context for the kernel figures, not a part of
    the metric; the libraries' first calls (kernel selection) are outside the timed regions."""
    import ctypes as C
    import torch.nn.functional as F
    dev = "cuda:0"
    cs = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    P = lambda t: C.c_void_p(t.data_ptr())
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def ms_of(fn, reps):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        best = float("inf")
        for _ in range(3):
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1) / reps)
        return best

    res = {}
    torch.backends.cuda.matmul.allow_tf32 = False
    for n in (4096, 8192):
        reps = 20 if n == 4096 else 4
        a, b = torch.randn(n, n, device=dev), torch.randn(n, n, device=dev)
        c = torch.empty(n, n, device=dev)
        ours = ms_of(lambda: mgb.check(mgb.mgb_gemm_f32_enqueue(cs, P(a), P(b), P(c), n, n, n), "gemm_f32"), reps)
        lib = ms_of(lambda: torch.matmul(a, b, out=c), reps)
        res["gemm_f32_%d" % n] = dict(unit="TFLOP/s", this_library=round(2.0 * n ** 3 / ours / 1e9, 1),
                                      torch_matmul=round(2.0 * n ** 3 / lib / 1e9, 1))
        ah, bh = a.bfloat16(), b.bfloat16()
        a16, b16 = ah.view(torch.int16), bh.view(torch.int16)
        ours = ms_of(lambda: mgb.check(mgb.mgb_gemm_bf16_enqueue(cs, P(a16), P(b16), P(c), n, n, n), "gemm_bf16"), reps * 4)
        ch = torch.empty(n, n, device=dev, dtype=torch.bfloat16)
        lib = ms_of(lambda: torch.matmul(ah, bh, out=ch), reps * 4)     # writes bf16, half the output bytes of ours
        res["gemm_bf16_%d" % n] = dict(unit="TFLOP/s", this_library=round(2.0 * n ** 3 / ours / 1e9, 1),
                                       torch_matmul_bf16_out=round(2.0 * n ** 3 / lib / 1e9, 1))
        log("vendor libraries: GEMM %d done" % n)
        del a, b, c, ah, bh, ch
    layers = W.cnn_layers()
    arr = (mgb.mgb_conv_layer * len(layers))(*[mgb.mgb_conv_layer(L["c_in"], L["c_out"], L["stride"]) for L in layers])
    wbits = W.cnn_weights(7, layers)
    for batch in (8, 1):
        mem, act, ob = C.c_uint64(), C.c_uint64(), C.c_uint64()
        g, blk = mgb.mgb_dim3(), mgb.mgb_dim3()
        mgb.check(mgb.mgb_cnn_probe(arr, len(layers), batch, 416, 416, C.byref(mem), C.byref(act), C.byref(ob),
                                    C.byref(g), C.byref(blk)), "mgb_cnn_probe")
        X = torch.from_numpy(W.cnn_input(7, batch).view("int16")).to(dev)
        Wd = [torch.from_numpy(x.view("int16")).to(dev) for x in wbits]
        ptrs = (C.c_void_p * len(Wd))(*[t.data_ptr() for t in Wd])
        a0 = torch.zeros(act.value // 2, dtype=torch.int16, device=dev)
        a1 = torch.zeros(act.value // 2, dtype=torch.int16, device=dev)
        out = torch.zeros(ob.value // 4, dtype=torch.float32, device=dev)
        ours = ms_of(lambda: mgb.check(mgb.mgb_cnn_enqueue(cs, arr, len(layers), P(X), ptrs, P(a0), P(a1), P(out),
                                                           batch, 416, 416), "mgb_cnn_enqueue"), 20)
        # the same tensors as torch sees them: NHWC activations = channels-last NCHW, KRSC filters = channels-last KCRS
        xt = X.view(torch.bfloat16).view(batch, 416, 416, 3).permute(0, 3, 1, 2)
        wt = [t.view(torch.bfloat16).view(L["c_out"], 3, 3, L["c_in"]).permute(0, 3, 1, 2) for t, L in zip(Wd, layers)]

        def chain():
            y = xt
            for wl, L in zip(wt, layers):
                y = F.relu(F.conv2d(y, wl, stride=L["stride"], padding=1))
            return y
        t0 = time.perf_counter()
        y = chain()
        torch.cuda.synchronize()
        setup = time.perf_counter() - t0
        ref = y.permute(0, 2, 3, 1).float().reshape(-1)
        diff = float((out - ref).norm() / ref.norm())
        lib = ms_of(chain, 20)
        flops = sum(2.0 * batch * L["h_out"] * L["w_out"] * L["c_out"] * 9 * L["c_in"] for L in layers)
        res["conv_chain_416_batch%d" % batch] = dict(unit="ms", this_library=round(ours, 4), torch_conv2d_relu=round(lib, 4),
                                                     this_library_tflops=round(flops / ours / 1e9, 1),
                                                     torch_tflops=round(flops / lib / 1e9, 1),
                                                     outputs_rel_diff=round(diff, 5), torch_first_call_s=round(setup, 1))
        log("vendor libraries: conv chain batch %d done" % batch)
    return res


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
    from paper_2107_08538_amd import harness, profsum
    import workloads as W

    native = args.harness == "native"
    on_stream = args.release == "stream"

    def run(sched, tasks, release_on_stream=False, **kw):
        fn = harness.run_mix_native if native else harness.run_mix
        return fn(sched, tasks, release_on_stream=release_on_stream, workers=args.workers, **kw)

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
    n_tasks = len(tasks)

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

    # measured operand-fetch and LDS-read rates (what the tile shapes of the MFMA kernels were chosen by):
    # bytes per clock and CU at the nominal 2.4 GHz; rows of 64 bytes are half cache lines
    rates = {}
    rsrc = torch.zeros(64 << 20, dtype=torch.uint8, device="cuda:0")
    rsink = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    nb = C.c_double(0.0)

    def rate(fn):
        fn()
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        return nb.value / (e0.elapsed_time(e1) / 1e3) / 256 / 2.4e9

    for label, foot, row in (("l2_rows_64B", 2 << 20, 64), ("l2_rows_128B", 2 << 20, 128),
                             ("llc_rows_64B", 64 << 20, 64), ("llc_rows_128B", 64 << 20, 128)):
        rates[label] = round(rate(lambda: mgb.check(mgb.mgb_fetch_rate_enqueue(
            cs, C.c_void_p(rsrc.data_ptr()), foot, row, 8192, 512, 500, C.c_void_p(rsink.data_ptr()), C.byref(nb)),
            "mgb_fetch_rate_enqueue")), 1)
    for label, swz in (("lds_fragment_reads_swizzled", 1), ("lds_fragment_reads_plain", 0)):
        rates[label] = round(rate(lambda: mgb.check(mgb.mgb_lds_read_rate_enqueue(
            cs, swz, 512, 1000, C.c_void_p(rsink.data_ptr()), C.byref(nb)), "mgb_lds_read_rate_enqueue")), 1)
    del rsrc

    pol = dict(hard=mgb.MGB_POLICY_HARD, soft=mgb.MGB_POLICY_SOFT, serial=mgb.MGB_POLICY_SERIAL)[args.policy]
    qm = dict(backfill=mgb.MGB_QUEUE_BACKFILL, fifo=mgb.MGB_QUEUE_FIFO)[args.queue]
    free_b, total_b = torch.cuda.mem_get_info()
    cap = min(spec["cap_bytes"], total_b)
    sched = mgb.Sched(policy=pol, queue_mode=qm, mem_cap_bytes=cap)

    log("inputs resident (%d tasks, %.1f s); stream copy %.0f GB/s; MFMA loop %.0f (f32) / %.0f (bf16) TFLOP/s"
        % (n_tasks, t_gen, copy_gbps, mfma_tflops["f32"], mfma_tflops["bf16"]))
    timed_kw = dict(release_on_stream=on_stream, use_arrivals=not args.batch)
    for _ in range(args.warmup):
        run(sched, tasks, **timed_kw)
    log("warm-up done, %d masked streams" % sched.stats().n_streams)
    # (the interpreter's cyclic collector would otherwise run a full collection of this process's large heap
    # once or twice inside the timed region, tens of milliseconds each, between two passes)
    gc.collect()
    gc.disable()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    runs = []
    for _ in range(args.steps):
        runs.append(run(sched, tasks, **timed_kw))
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    gc.enable()
    log("timed region done: %d steps in %.3f s, %d masked streams" % (args.steps, elapsed, sched.stats().n_streams))
    sums = [harness.summarize(r, m) for r, m in runs]
    value = n_tasks * args.steps / elapsed
    mean_turn = sum(s["mean_turnaround_ms"] for s in sums) / len(sums)
    if args.dump_records:
        with open(args.dump_records, "w") as f:
            json.dump([dict(task_id=r["task_id"], kind=r["kind"], granule_mask=int(r["record"].granule_mask),
                            gpu_start_ms=r["record"].gpu_start_ms, gpu_stop_ms=r["record"].gpu_stop_ms,
                            gpu_ms=r["record"].gpu_ms) for r in runs[-1][0] if r.get("record") is not None], f)

    # per-kernel figures from the timed region (HIP events bracket each task on its own stream)
    kern = {}
    for rec, _ in runs:
        for r, t in zip(rec, tasks):
            k = kern.setdefault(t.kernel_name, dict(ms=0.0, launches=0, tasks=0, bytes=0.0, flops=0.0, edges=0))
            launches = t.launches if t.launches is not None else max(1, int(t.depth.value))
            k["ms"] += r["gpu_ms"]; k["launches"] += launches; k["tasks"] += 1
            k["bytes"] += t.alg_bytes; k["flops"] += t.alg_flops; k["edges"] += t.edges
    dominant = max(kern, key=lambda n: kern[n]["ms"])

    def measured_ceiling(name):
        # what this device sustains on the same resource with nothing else in the way: the plain copy
        # kernel for HBM-bound kernels, the register-only MFMA loop of the kernel's dtype for the
        # matrix kernels (none for plain vector arithmetic)
        bound = PEAKS[name][0]
        if bound == "hbm":
            return copy_gbps
        if bound == "mfma":
            return mfma_tflops["f32" if name == "gemm_f32_dma_kernel" else "bf16"]
        return None

    def traffic_of(name):
        # HBM-side bytes per launch from the counter runs summarised under profiles/ (Mix-16 shapes
        # only), None once the kernel's source differs from the one that was measured
        return profsum.traffic_for(TRAFFIC_TABLE, name) if args.mix == "mix16" else None

    def roof(name, k):
        bound, peak, unit = PEAKS[name]
        secs = k["ms"] / 1e3
        work = k["bytes"] / 1e9 if bound == "hbm" else k["flops"] / 1e12
        ach = work / secs
        tr = traffic_of(name)
        out = dict(kernel=name, bound=bound, achieved=round(ach, 2), peak=round(peak, 1), unit=unit,
                   frac=round(ach / peak, 4), traffic=None if tr is None else round(tr),
                   avg_launch_us=round(1e3 * k["ms"] / k["launches"], 2), launches=k["launches"])
        ceil = measured_ceiling(name)
        if ceil:
            out["measured_ceiling"] = round(ceil, 1)
            out["frac_of_measured"] = round(ach / ceil, 4)
        if tr is not None:
            # the same launches against the HBM peak, from the counters
            out["hbm_counter_gbs"] = round(tr * k["launches"] / secs / 1e9, 1)
            out["hbm_counter_frac"] = round(tr * k["launches"] / secs / 1e9 / 8000.0, 4)
        if bound == "alu":
            # bonus figure: 8 bytes per cell update as if every sweep went through HBM (fused sweeps
            # move a fraction of that, so this may exceed the HBM peak and is no roofline fraction)
            out["one_sweep_per_pass_equivalent_gbs"] = round(k["bytes"] / 1e9 / secs, 1)
        if k["edges"]:
            out["gteps"] = round(k["edges"] / secs / 1e9, 2)      # stored directed edges per second of traversal
            # the same traversal if every 4-byte probe of a neighbour's state cost a whole 32-byte sector of
            # HBM (a model figure beside the algorithmic one: the level kernel probes a bitmap that it keeps
            # in LDS or L2, and its counter traffic stays near the algorithmic bytes)
            out["sector_granular_equivalent_gbs"] = round((k["bytes"] + 28.0 * k["edges"]) / secs / 1e9, 1)
        return out

    out = dict(metric="aggregate tasks/s through probe+admit+partition+launch+release (with mean turnaround, max slowdown)",
               value=round(value, 2), unit="tasks/s", n_gpus=1, steps=args.steps, warmup=args.warmup,
               ms_per_step=round(1e3 * elapsed / args.steps, 3), higher_is_better=True, scaling="weak",
               vs_baseline=None, dtype="f32", data="synthetic",
               config=dict(workload="%s: %s" % (spec["name"], ", ".join(sorted({t.kind for t in spec["tasks"]}))),
                           policy=args.policy, queue=args.queue, tasks=n_tasks, workers=min(n_tasks, args.workers or harness.MAX_WORKERS),
                           arrivals="all at t=0" if args.batch else "as the mix states", harness=args.harness,
                           release=args.release, cap_bytes=cap, granule_cus=int(sched.desc.granule_cus), n_cu=256),
               # `value` is over the whole timed region; the comparisons below (serialised run, other policies) are
               # medians of per-pass figures, so the per-pass median and what lies between the passes (the pool's
               # start and join, the records) are given too
               tasks_per_s_median_of_passes=round(med([s["tasks_per_s"] for s in sums]), 2),
               between_passes_ms=round(1e3 * (elapsed - sum(m for _, m in runs)) / args.steps, 3),
               mean_turnaround_ms=round(mean_turn, 3),
               median_turnaround_ms=round(med([s["mean_turnaround_ms"] for s in sums]), 3),
               mean_wait_ms=round(sum(s["mean_wait_ms"] for s in sums) / len(sums), 3),
               # admission - probe; with releases ordered on the stream a task can be admitted while its predecessor's
               # kernels still run, so the time a task spends not running (turnaround - its kernels' time: waiting
               # for admission, queued on the device behind its predecessor, hand-over) is given beside it
               mean_not_running_ms=round(sum(s["mean_turnaround_ms"] - s["gpu_busy_ms"] / max(1, s["tasks"]) for s in sums) / len(sums), 3),
               input_gen_s=round(t_gen, 1), stream_copy_gbps=round(copy_gbps, 1),
               mfma_loop_tflops={k: round(v, 1) for k, v in mfma_tflops.items()},
               bytes_per_clk_per_cu=rates)
    out["roofline"] = roof(dominant, kern[dominant])
    out["kernels"] = [roof(n, k) for n, k in kern.items() if n != dominant]

    if not args.no_extras:
        kinds = sorted({t.spec.kind for t in tasks})

        def per_task_median(passes):
            return [med([p[0][i]["gpu_ms"] for p in passes]) for i in range(n_tasks)]

        def slowdown(co, ref):
            s = [c / a - 1.0 for c, a in zip(co, ref) if a > 0 and c > 0]
            return dict(max_pct=round(100 * max(s), 2), mean_pct=round(100 * sum(s) / len(s), 2),
                        by_kind_max_pct={k: round(100 * max(x for x, t in zip(s, tasks) if t.spec.kind == k), 2) for k in kinds})

        # the same mix, serialised: one task at a time on all 256 CUs in arrival order, a task owning the
        # device until the host has seen it finish (single assignment, Sec. IV); same harness, same
        # warm-up, medians over the passes
        log("serialised comparator")
        ser = mgb.Sched(policy=mgb.MGB_POLICY_SERIAL, queue_mode=mgb.MGB_QUEUE_FIFO, mem_cap_bytes=cap)
        for _ in range(max(1, args.warmup)):
            run(ser, tasks, use_arrivals=not args.batch)
        sruns = [run(ser, tasks, use_arrivals=not args.batch) for _ in range(max(5, args.steps // 2))]
        ssum = [harness.summarize(r, m) for r, m in sruns]
        out["serialised_gpu"] = dict(tasks_per_s=round(med([s["tasks_per_s"] for s in ssum]), 2),
                                     mean_turnaround_ms=round(med([s["mean_turnaround_ms"] for s in ssum]), 3),
                                     passes=len(sruns), release="host")
        out["speedup_vs_serialised"] = dict(
            throughput=round(med([s["tasks_per_s"] for s in sums]) / out["serialised_gpu"]["tasks_per_s"], 4),
            turnaround=round(out["serialised_gpu"]["mean_turnaround_ms"] / med([s["mean_turnaround_ms"] for s in sums]), 4))
        # kernel slowdown as the paper defines it (Sec. V, kernel-slowdown table): GPU time of a task in
        # the shared run over the same task in the single-assignment run of the same workload; per task
        # the median over the passes
        co, sa = per_task_median(runs), per_task_median(sruns)
        sl = slowdown(co, sa)
        out["max_slowdown_pct"], out["mean_slowdown_pct"], out["slowdown_by_kind_pct"] = sl["max_pct"], sl["mean_pct"], sl["by_kind_max_pct"]
        out["corun_gpu_ms"] = {k: round(max(c for c, t in zip(co, tasks) if t.spec.kind == k), 4) for k in kinds}
        out["serialised_gpu_ms"] = {k: round(max(c for c, t in zip(sa, tasks) if t.spec.kind == k), 4) for k in kinds}
        # each task alone, back to back on a busy (clocked-up) device: on all 256 CUs (single assignment)
        # and in the partition its own probe is granted on an otherwise empty device
        log("tasks alone")
        alone256, alone_part = [], []
        for t in tasks:
            for sch, dst in ((ser, alone256), (sched, alone_part)):
                run(sch, [t], use_arrivals=False)
                dst.append(med([run(sch, [t], use_arrivals=False)[0][0]["gpu_ms"] for _ in range(5)]))
        out["alone_back_to_back_gpu_ms"] = {k: round(min(a for a, t in zip(alone256, tasks) if t.spec.kind == k), 4) for k in kinds}
        out["slowdown_vs_alone_on_256_cus"] = slowdown(co, alone256)
        out["slowdown_vs_alone_in_the_same_partition"] = slowdown(co, alone_part)
        # the dominant kernel's own speed: the same figure as `roofline`, from the back-to-back launches
        # (the timed region above has idle gaps between arrivals, and the clocks ramp after each)
        da = [(a, t) for a, t in zip(alone256, tasks) if t.kernel_name == dominant]
        if da:
            bound, peak, unit = PEAKS[dominant]
            work = sum((t.alg_bytes / 1e9 if bound == "hbm" else t.alg_flops / 1e12) for _, t in da)
            ach = work / (sum(a for a, _ in da) / 1e3)
            out["roofline_back_to_back"] = dict(kernel=dominant, bound=bound, achieved=round(ach, 2), peak=round(peak, 1),
                                                unit=unit, frac=round(ach / peak, 4))
            if measured_ceiling(dominant):
                out["roofline_back_to_back"]["frac_of_measured"] = round(ach / measured_ceiling(dominant), 4)

        # batch variant (all tasks queued at t = 0, the paper's setting): capacity rather than arrival bound
        def device_idle(rec):
            # device clock (the events around every task, no profiler in the way): time during which no
            # task's kernels were between their start and stop events, by the kind of task that ended before it
            iv = sorted((r["record"].gpu_start_ms, r["record"].gpu_stop_ms, r["kind"]) for r in rec if r.get("record") is not None)
            idle, end, prev = {}, iv[0][1], iv[0][2]
            for a, b, kind in iv[1:]:
                if a > end:
                    idle[prev] = idle.get(prev, 0.0) + (a - end)
                if b > end:
                    end, prev = b, kind
            return idle, end - iv[0][0]

        def batch_leg(sch, release_on_stream, passes=5):
            run(sch, tasks, use_arrivals=False, release_on_stream=release_on_stream)
            rr = [run(sch, tasks, use_arrivals=False, release_on_stream=release_on_stream) for _ in range(passes)]
            ss = [harness.summarize(r, m) for r, m in rr]
            idles = [device_idle(r) for r, _ in rr]
            return rr, dict(tasks_per_s=round(med([x["tasks_per_s"] for x in ss]), 2),
                            device_span_ms=round(med([sp for _, sp in idles]), 3),
                            device_idle_ms_after={k: round(med([i.get(k, 0.0) for i, _ in idles]), 4) for k in kinds},
                            mean_turnaround_ms=round(med([x["mean_turnaround_ms"] for x in ss]), 3),
                            mean_wait_ms=round(med([x["mean_wait_ms"] for x in ss]), 3),
                            makespan_ms=round(med([x["makespan_ms"] for x in ss]), 3),
                            gpu_busy_ms=round(med([x["gpu_busy_ms"] for x in ss]), 3),
                            tasks_per_s_min_max=[round(min(x["tasks_per_s"] for x in ss), 1), round(max(x["tasks_per_s"] for x in ss), 1)])

        log("batch at t=0")
        brun, b = batch_leg(sched, on_stream)
        bsrun, bs = batch_leg(ser, False)
        _, bs_stream = batch_leg(ser, True)
        _, b_host = batch_leg(sched, False)
        b["release"] = args.release
        b["serialised_tasks_per_s"], b["serialised_mean_turnaround_ms"] = bs["tasks_per_s"], bs["mean_turnaround_ms"]
        b["speedup_vs_serialised"] = round(b["tasks_per_s"] / bs["tasks_per_s"], 4)
        b["turnaround_speedup_vs_serialised"] = round(bs["mean_turnaround_ms"] / b["mean_turnaround_ms"], 4)
        # the same two schedulers with the release the other way round, so that what the stream-ordered
        # release buys and what the partitioning buys can be told apart
        b["host_release_tasks_per_s"] = b_host["tasks_per_s"]
        b["serialised_stream_release_tasks_per_s"] = bs_stream["tasks_per_s"]
        b["host_release_device_idle_ms_after"] = b_host["device_idle_ms_after"]
        b["serialised_device_idle_ms_after"] = bs["device_idle_ms_after"]
        b["slowdown_vs_serialised_batch"] = slowdown(per_task_median(brun), per_task_median(bsrun))
        # what the co-run sustains as a whole over the makespan: algorithmic bytes and flops of the tasks,
        # and HBM-side bytes from the hardware counters (bytes per launch of each kernel x its launches)
        mk = 1e-3 * b["makespan_ms"]
        b["corun_algorithmic_hbm_gbs"] = round(sum(t.alg_bytes for t in tasks) / mk / 1e9, 1)
        b["corun_tflops"] = round(sum(t.alg_flops for t in tasks) / mk / 1e12, 2)
        trs = [traffic_of(t.kernel_name) for t in tasks]
        if all(x is not None for x in trs):
            moved = sum(x * (t.launches if t.launches is not None else max(1, int(t.depth.value))) for x, t in zip(trs, tasks))
            b["corun_hbm_gbs"] = round(moved / mk / 1e9, 1)
            b["corun_hbm_frac_of_peak"] = round(moved / mk / 1e9 / 8000.0, 4)
            b["corun_hbm_source"] = "rocprofv3 FETCH_SIZE + WRITE_SIZE per launch (profiles/mix16_hbm_traffic.md) x launches / makespan"
        else:
            b["corun_hbm_gbs"] = None
        b["corun_mfma_frac_of_peak"] = round(sum(t.alg_flops for t in tasks if t.kernel_name == "gemm_f32_dma_kernel") / mk / 1e12 / 157.3, 4)
        # busy cycles of the matrix and vector pipes over the co-run, from the counters: each kernel's share
        # of busy cycles (rocprofv3 MfmaUtil / VALUBusy, taken per kernel) weighted by its share of the makespan
        if args.mix == "mix16":
            per_task = per_task_median(brun)
            for key, counter in (("corun_mfma_util_pct", "MfmaUtil"), ("corun_valu_busy_pct", "VALUBusy")):
                u = [profsum.utilisation_for(TRAFFIC_TABLE, t.kernel_name, counter) for t in tasks]
                b[key] = None if any(x is None for x in u) else round(sum(x * ms for x, ms in zip(u, per_task)) / b["makespan_ms"], 2)
        out["batch_t0"] = b

        # the other policies on the same mix: Alg. 3 analogue (overlapping masks), FIFO queue,
        # HARD with one workgroup per CU as the residency limit ("spread": a task gets as many
        # CUs as it has workgroups, so only tasks that cannot fill the device share it), and the
        # memory-blind CG baseline of Sec. IV at four jobs per device; kernel slowdown of each against
        # the single-assignment run
        sched.destroy()
        sched = None
        sweep = {}
        for name, pol2, q2, wgcu, ratio in (("soft_backfill", mgb.MGB_POLICY_SOFT, mgb.MGB_QUEUE_BACKFILL, 32, 8),
                                            ("hard_fifo", mgb.MGB_POLICY_HARD, mgb.MGB_QUEUE_FIFO, 32, 8),
                                            ("hard_spread", mgb.MGB_POLICY_HARD, mgb.MGB_QUEUE_BACKFILL, 1, 8),
                                            ("cg_ratio4", mgb.MGB_POLICY_CG, mgb.MGB_QUEUE_BACKFILL, 32, 4)):
            log("policy sweep: " + name)
            s2 = mgb.Sched(policy=pol2, queue_mode=q2, mem_cap_bytes=cap, max_wg_per_cu=wgcu, max_running=ratio)
            run(s2, tasks, release_on_stream=on_stream)
            aruns = [run(s2, tasks, release_on_stream=on_stream) for _ in range(3)]
            a = [harness.summarize(r, m) for r, m in aruns]
            bruns, bb = batch_leg(s2, on_stream)
            sweep[name] = dict(tasks_per_s=round(med([x["tasks_per_s"] for x in a]), 2),
                               mean_turnaround_ms=round(med([x["mean_turnaround_ms"] for x in a]), 3),
                               max_slowdown_pct=slowdown(per_task_median(aruns), sa)["max_pct"],
                               batch_tasks_per_s=bb["tasks_per_s"], batch_mean_turnaround_ms=bb["mean_turnaround_ms"],
                               batch_mean_wait_ms=bb["mean_wait_ms"],
                               batch_speedup_vs_serialised=round(bb["tasks_per_s"] / bs["tasks_per_s"], 4),
                               batch_max_slowdown_pct=slowdown(per_task_median(bruns), per_task_median(bsrun))["max_pct"])
            s2.destroy()
        out["other_policies"] = sweep
        ser.destroy()
        if not args.no_other_mixes and args.mix == "mix16":
            out["other_mixes"] = other_mixes(mgb, harness, W, run, total_b, on_stream)
        log("lazy runtime")
        out["lazy_runtime"] = lazy_leg(mgb, cap)
        log("multi-process front end")
        out["ipc_front_end"] = ipc_leg(mgb)
    if args.vendor_libraries:
        log("vendor libraries")
        out["vendor_libraries"] = vendor_libraries(torch, mgb, W, log)
    if not args.no_cpu_baseline:
        log("cpu baseline")
        out["cpu_baseline"] = cpu_baseline(spec)
    if sched is not None:
        sched.destroy()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
