"""Whole task mixes through the scheduler on the GPU: every output against the CPU checker, every
decision against the replay.  Mix-16 runs at its full size; CNN-8 and Mixed-128 run on reduced
instances that the serial checker can recompute in seconds."""
import numpy as np
import pytest

import oracle
import workloads as W
from helpers import (FREIVALDS_TOL, assert_trace_matches_replay, band_samples, check_ledger_invariants, cnn_patch_for,
                     freivalds_ratio, frobenius_rel, verify_task_output, verify_task_output_at_full_size)

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

import paper_2107_08538_amd as mgb  # noqa: E402
from paper_2107_08538_amd import harness  # noqa: E402


def _run(spec, use_arrivals=True, time_scale=1.0, release_on_stream=False, **sched_kw):
    data = [W.task_data(t) for t in spec["tasks"]]
    tasks = [harness.build_task(t, d) for t, d in zip(spec["tasks"], data)]
    cap = min(spec["cap_bytes"], torch.cuda.mem_get_info()[1])
    s = mgb.Sched(mem_cap_bytes=cap, **sched_kw)
    rec, makespan = harness.run_mix(s, tasks, use_arrivals=use_arrivals, time_scale=time_scale,
                                    release_on_stream=release_on_stream)
    return s, tasks, data, rec


def _assert_one_owner_in_device_time(rec, exclusive=True):
    """Tasks whose granule sets overlap must not overlap on the device clock (the events around
    each task's kernels, read against the scheduler's clock origin)."""
    iv = sorted((r["record"].gpu_start_ms, r["record"].gpu_stop_ms, r["record"].granule_mask, r["task_id"])
                for r in rec if not r.get("crashed"))
    pairs = 0
    for i, (a0, a1, am, aid) in enumerate(iv):
        assert a1 >= a0 > 0.0
        for b0, b1, bm, bid in iv[i + 1:]:
            if am & bm:
                pairs += 1
                if exclusive:
                    assert b0 >= a1 - 2e-3, ("tasks %d and %d share granules and overlap in time" % (aid, bid), a0, a1, b0, b1)
    return pairs


@pytest.mark.parametrize("policy", [mgb.MGB_POLICY_HARD, mgb.MGB_POLICY_SERIAL])
def test_mix16_batch_released_on_stream_outputs_decisions_and_device_time(policy):
    # every task hands its granules and bytes back when its last kernel is enqueued; its successor
    # is launched behind its stop event.  Outputs, decisions and the ledger are what they are with
    # host-observed releases, and on the device no two tasks that share granules overlap.
    s, tasks, data, rec = _run(W.mix16(seed=3), use_arrivals=False, release_on_stream=True, policy=policy,
                               max_running=16)
    for t, d in zip(tasks, data):
        # (Jacobi through the dependency cones of sampled cells here; in full in test_mix16_full_size_...)
        (verify_task_output_at_full_size if t.spec.kind == "jacobi" else verify_task_output)(t, d)
    trace = s.trace()
    dec = assert_trace_matches_replay(s.desc, trace)
    check_ledger_invariants(s.desc, trace)
    assert (dec["kind"] == oracle.D_ADMIT).sum() == 16
    assert _assert_one_owner_in_device_time(rec) == 16 * 15 // 2          # every task asks for the whole device
    sm = harness.summarize(rec, 0.0)
    assert sm["tasks"] == 16 and sm["gpu_busy_ms"] <= sm["makespan_ms"] * 1.001
    assert s.destroy() == 0


@pytest.mark.parametrize("release_on_stream", [False, True])
def test_mix16_and_cnn8_through_the_native_worker_pool(release_on_stream):
    # the same jobs through mgb_pool_run (probe derivation, wait, launch, release inside the library)
    for spec, kw in ((W.mix16(seed=5), dict(use_arrivals=False)), (W.cnn8(h=52, w=52), dict(time_scale=0.1))):
        data = [W.task_data(t) for t in spec["tasks"]]
        tasks = [harness.build_task(t, d) for t, d in zip(spec["tasks"], data)]
        s = mgb.Sched(mem_cap_bytes=min(spec["cap_bytes"], torch.cuda.mem_get_info()[1]))
        rec, _ = harness.run_mix_native(s, tasks, release_on_stream=release_on_stream, **kw)
        for t, d in zip(tasks, data):
            (verify_task_output_at_full_size if t.spec.kind == "jacobi" else verify_task_output)(t, d)
        trace = s.trace()
        assert_trace_matches_replay(s.desc, trace)
        check_ledger_invariants(s.desc, trace)
        _assert_one_owner_in_device_time(rec)
        sm = harness.summarize(rec, 0.0)
        assert sm["tasks"] == len(tasks) and sm["crashed"] == 0 and sm["tasks_per_s"] > 0
        for r, t in zip(rec, tasks):
            assert (r["record"].mem_bytes, r["granules"]) == (t.mem, -(-min(256, -(-t.grid.x // max(1, min(32 // -(-t.block.x // 64), t.wg_per_cu)))) // 32))
        assert s.destroy() == 0


@pytest.mark.parametrize("policy,ratio", [(mgb.MGB_POLICY_SOFT, 8), (mgb.MGB_POLICY_CG, 4)])
def test_mix16_pool_with_overlapping_policies_released_on_stream(policy, ratio):
    # Alg. 3's analogue and the ratio baseline let tasks share CUs, so a release on the stream orders
    # nothing for compute (and memory never binds at 288 GB): tasks do overlap in device time, and every
    # output and decision is still what the checker says
    spec = W.mix16(seed=7)
    data = [W.task_data(t) for t in spec["tasks"]]
    tasks = [harness.build_task(t, d) for t, d in zip(spec["tasks"], data)]
    s = mgb.Sched(mem_cap_bytes=min(spec["cap_bytes"], torch.cuda.mem_get_info()[1]), policy=policy, max_running=ratio)
    rec, _ = harness.run_mix_native(s, tasks, use_arrivals=False, release_on_stream=True)
    for t, d in zip(tasks, data):
        (verify_task_output_at_full_size if t.spec.kind == "jacobi" else verify_task_output)(t, d)
    assert_trace_matches_replay(s.desc, s.trace())
    if policy != mgb.MGB_POLICY_CG:                                       # (CG shares the whole-device mask by definition)
        check_ledger_invariants(s.desc, s.trace())
    iv = sorted((r["record"].gpu_start_ms, r["record"].gpu_stop_ms) for r in rec)
    assert any(b0 < a1 for (a0, a1), (b0, b1) in zip(iv, iv[1:]))         # some tasks did run at the same time
    assert harness.summarize(rec, 0.0)["tasks"] == 16
    assert s.destroy() == 0


def test_mixed128_reduced_released_on_stream_partitions_keep_one_owner():
    # small tasks share the device in disjoint partitions; a partition changes hands on the device
    s, tasks, data, rec = _run(W.mixed128(shrink=4), use_arrivals=False, release_on_stream=True)
    for t, d in zip(tasks, data):
        if t.spec.kind != "jacobi" or t.spec.params["n"] <= 1024:      # (the serial checker's time)
            verify_task_output(t, d)
    trace = s.trace()
    assert_trace_matches_replay(s.desc, trace)
    check_ledger_invariants(s.desc, trace)
    sizes = {bin(r["record"].granule_mask).count("1") for r in rec}
    assert sizes == {1, 2, 4, 8}                                     # eighths ... the whole device
    assert _assert_one_owner_in_device_time(rec) > 128
    assert s.destroy() == 0


def test_mix16_full_size_outputs_and_decisions():
    s, tasks, data, rec = _run(W.mix16())
    assert sorted(t.spec.kind for t in tasks).count("jacobi") >= 1
    for t, d in zip(tasks, data):
        verify_task_output(t, d)
    trace = s.trace()
    dec = assert_trace_matches_replay(s.desc, trace)
    check_ledger_invariants(s.desc, trace)
    assert (dec["kind"] == oracle.D_ADMIT).sum() == 16
    # demand the probes carried: GEMM 4096^3, BFS 2^20 (256 workgroups, one per CU because each keeps
    # the 128 KiB frontier bitmap in LDS) and Jacobi 4096^2 (504 workgroups of long-running waves, two
    # per CU) = the whole device (8 granules of 32 CUs)
    want = {"gemm_f32": 8, "jacobi": 8, "bfs": 8}
    for r, t in zip(rec, tasks):
        assert r["granules"] == want[t.spec.kind]
    assert s.destroy() == 0


@pytest.mark.parametrize("policy", [mgb.MGB_POLICY_HARD, mgb.MGB_POLICY_SOFT, mgb.MGB_POLICY_SERIAL])
def test_mix16_batch_at_t0_all_policies(policy):
    # all 16 probes issued before anything runs (the paper's batch setting): queues must form
    s, tasks, data, rec = _run(W.mix16(seed=3), use_arrivals=False, policy=policy, max_running=16)
    for t, d in zip(tasks, data):
        if t.spec.kind != "jacobi":             # Jacobi is covered at full size above
            verify_task_output(t, d)
    trace = s.trace()
    dec = assert_trace_matches_replay(s.desc, trace)
    check_ledger_invariants(s.desc, trace)
    waits = (dec["kind"] == oracle.D_WAIT).sum()
    if policy == mgb.MGB_POLICY_SERIAL:
        assert waits == 15
    elif policy == mgb.MGB_POLICY_HARD:
        assert waits > 0
    else:
        assert waits == 0                       # memory never binds here and compute is soft
    assert s.destroy() == 0


def test_memory_blind_ratio_packing_loses_jobs_that_admission_control_finishes():
    # Sec. V-B's contrast on a memory-tight mix: packing by a fixed jobs-per-device ratio without
    # looking at footprints loses jobs to out-of-memory, the probe-driven ledger finishes all.
    spec = W.pressure32(seed=9, scale=1 / 32)
    data = [W.task_data(t) for t in spec["tasks"]]
    tasks = [harness.build_task(t, d) for t, d in zip(spec["tasks"], data)]
    cap = spec["cap_bytes"]
    cg = mgb.Sched(policy=mgb.MGB_POLICY_CG, max_running=32, mem_cap_bytes=cap)
    rec, mk = harness.run_mix(cg, tasks, use_arrivals=False)
    lost = [r for r in rec if r.get("crashed")]
    assert 0 < len(lost) < 32
    trace = cg.trace()
    dec = assert_trace_matches_replay(cg.desc, trace)
    assert ((dec["kind"] == oracle.D_REJECT) & (dec["code"] == mgb.MGB_E_OOM)).sum() == len(lost)
    done = {r["task_id"] for r in rec if not r.get("crashed")}
    for t, d in zip(tasks, data):
        if t.spec.task_id in done:
            verify_task_output(t, d)
    assert harness.summarize(rec, mk)["crashed"] == len(lost)
    assert cg.destroy() == 0
    s = mgb.Sched(policy=mgb.MGB_POLICY_HARD, mem_cap_bytes=cap)
    rec, mk = harness.run_mix(s, tasks, use_arrivals=False)
    assert not any(r.get("crashed") for r in rec) and harness.summarize(rec, mk)["tasks"] == 32
    check_ledger_invariants(s.desc, s.trace())
    assert s.destroy() == 0


def test_cnn8_reduced_images():
    s, tasks, data, rec = _run(W.cnn8(h=52, w=52), time_scale=0.1)
    assert {t.spec.params["batch"] for t in tasks} <= {1, 2, 4, 8}
    for t, d in zip(tasks, data):
        verify_task_output(t, d)
    trace = s.trace()
    assert_trace_matches_replay(s.desc, trace)
    check_ledger_invariants(s.desc, trace)
    assert s.destroy() == 0


def test_mixed128_reduced_sizes():
    spec = W.mixed128(shrink=16)
    kinds = {t.kind for t in spec["tasks"]}
    assert kinds == {"jacobi", "gemm_f32", "gemm_bf16", "bfs"} and len(spec["tasks"]) == 128
    s, tasks, data, rec = _run(spec, time_scale=0.25)
    for t, d in zip(tasks, data):
        verify_task_output(t, d)
    trace = s.trace()
    dec = assert_trace_matches_replay(s.desc, trace)
    check_ledger_invariants(s.desc, trace)
    assert (dec["kind"] == oracle.D_ADMIT).sum() == 128
    grids = sorted(int(r["grid"][0]) for r in trace if r["kind"] == mgb.MGB_EV_PROBE)
    assert grids[0] == 8 and grids[-1] > grids[0]     # a range of small grids that share the device
    assert s.destroy() == 0


def test_mixed128_full_size_every_output_verified():
    """All 128 tasks at the sizes the mix states (Jacobi side and GEMM dimension 1024 - 8192, BFS on
    2^16 - 2^22 vertices), queued at t = 0 and run as the bench runs them (worker pool inside the
    library, releases ordered on the device).  Every output is checked: BFS levels in full, Jacobi on
    the dependency cones of sampled cells, every GEMM on one sample per 64 x 64 block of C and by
    Freivalds' check of the whole product.  Decisions replay; partitions keep one owner in device time."""
    from concurrent.futures import ThreadPoolExecutor
    spec = W.mixed128()
    with ThreadPoolExecutor(max_workers=16) as ex:
        data = list(ex.map(W.task_data, spec["tasks"]))
    print("mixed128 full: inputs drawn", flush=True)
    tasks = [harness.build_task(t, d) for t, d in zip(spec["tasks"], data)]
    s = mgb.Sched(mem_cap_bytes=min(spec["cap_bytes"], torch.cuda.mem_get_info()[1]))
    rec, _ = harness.run_mix_native(s, tasks, use_arrivals=False, release_on_stream=True)
    print("mixed128 full: mix ran", flush=True)
    with ThreadPoolExecutor(max_workers=16) as ex:                   # the checker's calls release the interpreter lock
        ratios = list(ex.map(lambda td: verify_task_output_at_full_size(*td), zip(tasks, data)))
    ratios = [r for r in ratios if r is not None]
    print("mixed128 full: %d GEMMs, largest Freivalds ratio %.3g (tolerance %.1g)" % (len(ratios), max(ratios), FREIVALDS_TOL), flush=True)
    assert len(ratios) == sum(t.spec.kind.startswith("gemm") for t in tasks) == 40
    trace = s.trace()
    dec = assert_trace_matches_replay(s.desc, trace)
    check_ledger_invariants(s.desc, trace)
    assert (dec["kind"] == oracle.D_ADMIT).sum() == 128 and (dec["kind"] == oracle.D_WAIT).sum() > 64
    _assert_one_owner_in_device_time(rec)
    # the launch geometries the probes carried span two orders of magnitude (24 workgroups for the
    # smallest traversal ... 3488 for the largest stencil) and every partition size from an eighth of
    # the device to all of it is asked for, so small tasks do share the device
    grids = sorted(int(r["grid"][0]) for r in trace if r["kind"] == mgb.MGB_EV_PROBE)
    assert grids[0] <= 32 and grids[-1] >= 2048 and grids[-1] >= 100 * grids[0]
    assert {bin(r["record"].granule_mask).count("1") for r in rec} == {1, 2, 4, 8}
    assert s.destroy() == 0


def test_cnn8_full_size_in_the_mix_sampled_output_pixels():
    """The eight 10-layer nets on 416 x 416 images at the batch sizes the mix draws, queued at t = 0
    through the worker pool.  The fp32 output (batch x 13 x 13 x 512) is checked on sampled pixels:
    each is recomputed by the serial checker's whole chain (bf16 rounding between layers included)
    from the window of the input image that decides it."""
    from concurrent.futures import ThreadPoolExecutor
    spec = W.cnn8()
    data = [W.task_data(t) for t in spec["tasks"]]
    tasks = [harness.build_task(t, d) for t, d in zip(spec["tasks"], data)]
    assert {t.spec.params["batch"] for t in tasks} <= {1, 2, 4, 8} and len({t.spec.params["batch"] for t in tasks}) >= 3
    s = mgb.Sched(mem_cap_bytes=min(spec["cap_bytes"], torch.cuda.mem_get_info()[1]))
    rec, _ = harness.run_mix_native(s, tasks, use_arrivals=False, release_on_stream=True)
    jobs = []
    for t, d in zip(tasks, data):
        b = t.spec.params["batch"]
        rng = np.random.default_rng(100 + t.spec.task_id)
        got = t.tensors["out"].cpu().numpy().reshape(b, 13, 13, 512)
        strides = [L["stride"] for L in d["layers"]]
        pix = [(b - 1, 0, 0), (0, 12, 12), (int(rng.integers(0, b)), int(rng.integers(0, 13)), int(rng.integers(0, 13))),
               (int(rng.integers(0, b)), 12, int(rng.integers(0, 13)))]
        for (bi, oy, ox) in pix:
            jobs.append((t.spec.task_id, d, strides, got[bi, oy, ox].astype(np.float64), bi, oy, ox))

    def one(job):
        tid, d, strides, got, bi, oy, ox = job
        y0, y1, x0, x1, ly, lx = cnn_patch_for(oy, ox, 416, 416)
        ref = oracle.cnn_forward(np.ascontiguousarray(d["x"][bi:bi + 1, y0:y1, x0:x1, :]), d["weights"], strides)[0, ly, lx]
        return tid, frobenius_rel(got, ref), float(np.abs(ref).max())
    with ThreadPoolExecutor(max_workers=16) as ex:
        res = list(ex.map(one, jobs))
    worst = max(r[1] for r in res)
    print("cnn8 full: %d output pixels x 512 channels, worst relative Frobenius error %.3g" % (len(res), worst), flush=True)
    assert worst <= 1e-2 and all(r[2] > 0 for r in res)              # (a pixel of zeros would prove nothing)
    trace = s.trace()
    assert_trace_matches_replay(s.desc, trace)
    check_ledger_invariants(s.desc, trace)
    _assert_one_owner_in_device_time(rec)
    assert s.destroy() == 0


def test_pressure32_full_size_sampled():
    """16 fp32 GEMM 32768^3 (12 GiB each) + 16 Jacobi 16384^2 x50 (2 GiB each), all at t = 0, cap =
    summed footprints / 1.5 so that admission has to queue.  Inputs of this size are drawn on the
    device (seeded torch generator); outputs are checked on sampled entries that the serial checker
    recomputes one by one from rows / columns / patches copied back to the host."""
    import ctypes as C
    spec = W.pressure32(seed=5)
    free_b, total_b = torch.cuda.mem_get_info()
    need = sum(16 * 3 * 32768 * 32768 * 4 for _ in (0,)) + 16 * 2 * 16384 * 16384 * 4
    if free_b < need + (8 << 30):
        pytest.skip("device has less free memory than the 224 GiB the mix needs")
    gen = torch.Generator(device="cuda:0")
    rng = np.random.default_rng(7)
    tasks, checks = [], {}
    P = lambda t: C.c_void_p(t.data_ptr())
    for t in spec["tasks"]:
        gen.manual_seed(t.seed % (2 ** 63))
        if t.kind == "gemm_f32":
            n = t.params["n"]
            A = torch.randn(n, n, device="cuda:0", generator=gen)
            B = torch.randn(n, n, device="cuda:0", generator=gen)
            Cc = torch.empty(n, n, device="cuda:0")
            probe = mgb.probe_of(mgb.mgb_gemm_f32_probe, n, n, n)
            assert probe[0] == 12 * 2 ** 30
            fn = (lambda A, B, Cc, n: lambda st: mgb.mgb_gemm_f32_enqueue(st, P(A), P(B), P(Cc), n, n, n))(A, B, Cc, n)
            # one row per band of 256 rows and one column per band of 256 columns: the 128 x 128 = 16384
            # entries at their crossings put a sample into every 256 x 256 tile of C
            rows, cols = band_samples(n, n, 256, 1000 + t.task_id)
            rows[0], cols[-1] = 0, n - 1
            dev_r, dev_c = torch.from_numpy(rows).to("cuda:0"), torch.from_numpy(cols).to("cuda:0")
            checks[t.task_id] = ("gemm", A[dev_r].cpu().numpy(), B[:, dev_c].contiguous().cpu().numpy(), rows, cols)
            tasks.append(harness.Task(t, dict(A=A, B=B, C=Cc), probe, fn, "gemm_f32_dma_kernel", 1))
        else:
            n, it = t.params["n"], t.params["iters"]
            u0 = torch.rand(n, n, device="cuda:0", generator=gen)
            u0[0, :] = 0
            u0[-1, :] = 0
            u0[:, 0] = 0
            u0[:, -1] = 0
            u1 = u0.clone()
            probe = mgb.probe_of(mgb.mgb_jacobi_probe, n, it)
            assert probe[0] == 2 * 2 ** 30
            fn = (lambda u0, u1, n, it: lambda st: mgb.mgb_jacobi_enqueue(st, P(u0), P(u1), n, it))(u0, u1, n, it)
            # a cell after `it` sweeps depends on the initial cells within distance `it`: keep those patches
            pts = [(1, 1), (n - 2, n - 2), (1, n // 2), (int(rng.integers(60, n - 60)), int(rng.integers(60, n - 60))),
                   (int(rng.integers(1, n - 1)), int(rng.integers(1, n - 1)))]
            patches = []
            side = min(n, 2 * it + 3)                 # square window, shifted (not clipped) at the grid's rim
            for (r, c) in pts:
                r0 = min(max(0, r - it - 1), n - side)
                c0 = min(max(0, c - it - 1), n - side)
                patches.append((r, c, r0, c0, u0[r0:r0 + side, c0:c0 + side].cpu().numpy().copy()))
            checks[t.task_id] = ("jacobi", patches, it)
            tasks.append(harness.Task(t, dict(u0=u0, u1=u1), probe, fn, "jacobi", 1))
    s = mgb.Sched(mem_cap_bytes=spec["cap_bytes"])
    rec, makespan = harness.run_mix(s, tasks, use_arrivals=False)
    for t in tasks:
        kind = checks[t.spec.task_id][0]
        if kind == "gemm":
            _, a_rows, b_cols, rows, cols = checks[t.spec.task_id]
            dev_r, dev_c = torch.from_numpy(rows).to("cuda:0"), torch.from_numpy(cols).to("cuda:0")
            got = t.tensors["C"][dev_r][:, dev_c].cpu().numpy().astype(np.float64).ravel()
            ri, ci = np.meshgrid(np.arange(len(rows), dtype=np.uint32), np.arange(len(cols), dtype=np.uint32), indexing="ij")
            ref, den = oracle.gemm_f32_entries(a_rows, b_cols, ri.ravel(), ci.ravel())
            assert len(ref) == 16384 and (np.abs(got - ref) / den).max() <= 1e-4, t.spec.task_id
        else:
            _, patches, it = checks[t.spec.task_id]
            res = t.tensors["u0"] if it % 2 == 0 else t.tensors["u1"]
            for (r, c, r0, c0, patch) in patches:
                # the window's rim is held fixed by the checker, which is only true where it is the grid's
                # own ring; elsewhere the rim is at least it + 1 cells from (r, c), out of reach in `it` sweeps
                want = oracle.jacobi_f32(np.ascontiguousarray(patch), it)[r - r0, c - c0]
                assert float(res[r, c]) == float(want), (t.spec.task_id, r, c)
    # Freivalds' check of two whole 32768^3 products on the host (A, B, C copied back: 12 GiB each)
    gemms = [t for t in tasks if t.spec.kind == "gemm_f32"]
    for t in (gemms[0], gemms[-1]):
        ratio = freivalds_ratio(t.tensors["A"].cpu().numpy(), t.tensors["B"].cpu().numpy(), t.tensors["C"].cpu().numpy(), t.spec.task_id)
        print("pressure32: task %d Freivalds ratio %.3g (tolerance %.1g)" % (t.spec.task_id, ratio, FREIVALDS_TOL), flush=True)
        assert ratio <= FREIVALDS_TOL, (t.spec.task_id, ratio)
    trace = s.trace()
    dec = assert_trace_matches_replay(s.desc, trace)
    check_ledger_invariants(s.desc, trace)
    assert (dec["kind"] == oracle.D_WAIT).sum() > 0 and (dec["kind"] == oracle.D_ADMIT).sum() == 32
    assert trace["free_bytes"].min() >= 0 and trace["free_bytes"].max() <= spec["cap_bytes"]
    # worst wait: every GEMM (whole device) runs alone, so the last GEMM admitted waited for the 15 before it
    waits = [r["admit"] - r["probe"] for r in rec]
    assert max(waits) > 0
    assert s.destroy() == 0
