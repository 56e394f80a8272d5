"""The scheduler with the HIP backend: CU-masked placements, end-to-end Mix-4, trace replay."""
import ctypes as C
import threading

import numpy as np
import pytest

import oracle
import workloads as W
from helpers import assert_trace_matches_replay

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

import paper_2107_08538_amd as mgb  # noqa: E402

DEV = "cuda:0"


def P(t):
    return C.c_void_p(t.data_ptr())


def _where(stream, n_blocks=4096):
    out = torch.zeros(n_blocks, dtype=torch.int32, device=DEV)
    assert mgb.mgb_cu_trace_enqueue(stream, P(out), n_blocks) == 0
    torch.cuda.synchronize()
    return set(out.cpu().numpy().tolist())


def test_whole_device_policies_create_one_stream():
    # SERIAL and CG only ever grant the whole device: one masked stream, not the seven of HARD
    for kw in (dict(policy=mgb.MGB_POLICY_SERIAL), dict(policy=mgb.MGB_POLICY_CG, max_running=4)):
        s = mgb.Sched(**kw)
        assert s.stats().n_streams == 1
        rc, pl = s.probe(1, 1 << 20, (8, 1, 1), (64, 1, 1))
        assert rc == mgb.MGB_OK and pl.granule_mask == 0xFF and pl.stream
        assert s.complete(pl.ticket) == mgb.MGB_OK and s.stats().n_streams == 1
        assert s.destroy() == 0


def test_default_partitions_are_eighths_of_the_device():
    s = mgb.Sched()
    assert s.desc.granule_cus == 32 and s.stats().n_streams == 7      # whole, halves, quarters created up front
    pls = []
    for i, wgs in enumerate((8, 512, 1024, 100000)):                  # 1, 64, 128, 256 CUs at 8 workgroups per CU
        rc, pl = s.probe(i, 1 << 20, (wgs, 1, 1), (256, 1, 1))
        pls.append((rc, pl))
    assert [rc for rc, _ in pls] == [mgb.MGB_OK, mgb.MGB_OK, mgb.MGB_OK, mgb.MGB_WAIT]
    assert [pl.n_granules for _, pl in pls] == [1, 2, 4, 8]
    assert [pl.granule_mask for _, pl in pls[:3]] == [0x01, 0x0C, 0xF0]
    sets = [_where(pl.stream) for _, pl in pls[:3]]
    assert [len(x) for x in sets] == [32, 64, 128]
    for cus in sets:
        assert len(set(np.bincount([c >> 8 for c in cus], minlength=8))) == 1     # the same share of every XCD
    assert not (sets[0] & sets[1]) and not (sets[1] & sets[2]) and not (sets[0] & sets[2])
    assert s.stats().n_streams == 8                                   # only the one-eighth mask was new
    assert s.cancel(pls[3][1].ticket) == 0
    for _, pl in pls[:3]:
        assert s.complete(pl.ticket) == 0
    assert_trace_matches_replay(s.desc, s.trace())
    assert s.destroy() == 0


def test_placements_are_disjoint_sets_of_physical_cus():
    s = mgb.Sched(granule_cus=8)                                      # the finest partition: one CU per XCD
    pls = []
    for i, wgs in enumerate((512, 64, 1024, 8)):                      # 8, 1, 16, 1 granules
        rc, pl = s.probe(i, 1 << 20, (wgs, 1, 1), (256, 1, 1))
        assert rc == mgb.MGB_OK and pl.stream
        pls.append(pl)
    assert [pl.n_granules for pl in pls] == [8, 1, 16, 1]
    sets = [_where(pl.stream) for pl in pls]
    for pl, cus in zip(pls, sets):
        assert len(cus) == 8 * pl.n_granules                          # one CU per XCD per granule
        per_xcd = np.bincount([c >> 8 for c in cus], minlength=8)
        assert np.all(per_xcd == pl.n_granules)
    for i in range(4):
        for j in range(i + 1, 4):
            assert not (sets[i] & sets[j])                            # disjoint masks, disjoint CUs
    assert len(_where(None)) == 256                                   # an unmasked stream reaches all CUs
    for pl in pls:
        assert s.complete(pl.ticket) == 0
    rc, pl = s.probe(9, 1, (512, 1, 1), (256, 1, 1))                  # streams are cached per mask
    assert pl.granule_mask == pls[0].granule_mask and pl.stream == pls[0].stream
    assert s.stats().n_streams == 9      # 7 created up front (whole, halves, quarters) + two single granules
    assert s.complete(pl.ticket) == 0
    assert s.destroy() == 0


def _mix4_buffers(spec):
    bufs = {}
    for t in spec["tasks"]:
        if t.kind == "jacobi":
            u = W.jacobi_field(t.seed + t.task_id, t.params["n"])
            u0 = torch.from_numpy(u).to(DEV)
            bufs[t.task_id] = dict(host=u, u0=u0, u1=u0.clone())
        else:
            a, b = W.gemm_operands_f32(t.seed + t.task_id, t.params["m"], t.params["n"], t.params["k"])
            bufs[t.task_id] = dict(a=a, b=b, A=torch.from_numpy(a).to(DEV), B=torch.from_numpy(b).to(DEV),
                                   C=torch.zeros(t.params["m"], t.params["n"], device=DEV))
    return bufs


def test_mix4_end_to_end_matches_checker_and_replay():
    spec = W.mix4(seed=4)
    s = mgb.Sched(mem_cap_bytes=spec["cap_bytes"])
    bufs = _mix4_buffers(spec)
    torch.cuda.synchronize()
    errors, placed = [], {}

    def worker(t):
        try:
            b = bufs[t.task_id]
            if t.kind == "jacobi":
                mem, grid, block = mgb.probe_of(mgb.mgb_jacobi_probe, t.params["n"], t.params["iters"])
                assert mem == b["u0"].numel() * 4 * 2                 # footprint = sum of allocations
                fn = lambda st: mgb.mgb_jacobi_enqueue(st, P(b["u0"]), P(b["u1"]), t.params["n"], t.params["iters"])
            else:
                m, n, k = t.params["m"], t.params["n"], t.params["k"]
                mem, grid, block = mgb.probe_of(mgb.mgb_gemm_f32_probe, m, n, k)
                assert mem == (b["A"].numel() + b["B"].numel() + b["C"].numel()) * 4
                fn = lambda st: mgb.mgb_gemm_f32_enqueue(st, P(b["A"]), P(b["B"]), P(b["C"]), m, n, k)
            rc, pl = s.probe(t.task_id, mem, grid, block)
            if rc == mgb.MGB_WAIT:
                rc, pl = s.wait(pl.ticket)
            assert rc == mgb.MGB_OK and pl.stream
            placed[t.task_id] = (pl.granule_mask, pl.n_granules)
            assert s.launch(pl.ticket, fn) == 0
            rc, ms = s.sync(pl.ticket)
            assert rc == 0 and ms > 0
            assert s.complete(pl.ticket) == 0
        except Exception as e:  # noqa: BLE001
            errors.append((t.task_id, e))

    threads = [threading.Thread(target=worker, args=(t,)) for t in spec["tasks"]]
    for th in threads:
        th.start()
    for th in threads:
        th.join(timeout=100)
    assert not errors, errors
    torch.cuda.synchronize()
    for t in spec["tasks"]:
        b = bufs[t.task_id]
        if t.kind == "jacobi":
            it = t.params["iters"]
            got = (b["u0"] if it % 2 == 0 else b["u1"]).cpu().numpy()
            assert np.array_equal(got, oracle.jacobi_f32(b["host"], it))
            ref = oracle.jacobi_f64(b["host"], it)
            assert (np.abs(got - ref)[1:-1, 1:-1] / ref[1:-1, 1:-1]).max() <= 1e-5
        else:
            got = b["C"].cpu().numpy().astype(np.float64)
            ref, den = oracle.gemm_f32(b["a"], b["b"]), oracle.gemm_abs_f32(b["a"], b["b"])
            assert (np.abs(got - ref) / den).max() <= 1e-4
    # every task is small: one granule each, all four resident together
    assert all(g == 1 for _, g in placed.values())
    trace = s.trace()
    dec = assert_trace_matches_replay(s.desc, trace)
    assert (dec["kind"] == oracle.D_ADMIT).sum() == 4 and (dec["kind"] == oracle.D_WAIT).sum() == 0
    assert s.stats().free_bytes == spec["cap_bytes"]
    assert s.destroy() == 0


def test_memory_pressure_queues_and_worst_wait_matches_replay():
    # scaled-down pressure mix: summed footprints = 1.5 x cap, so admission must queue
    spec = W.pressure32(seed=3, scale=1 / 32)
    s = mgb.Sched(mem_cap_bytes=spec["cap_bytes"])
    errors = []
    bufs = {}
    for t in spec["tasks"]:
        if t.kind == "jacobi":
            n = t.params["n"]
            u0 = torch.from_numpy(W.jacobi_field(t.seed, n)).to(DEV)
            bufs[t.task_id] = (u0, u0.clone())
        else:
            n = t.params["n"]
            bufs[t.task_id] = (torch.randn(n, n, device=DEV), torch.randn(n, n, device=DEV),
                               torch.zeros(n, n, device=DEV))
    torch.cuda.synchronize()
    # all 32 tasks arrive at t = 0: their probes are issued back to back in task-id order before
    # anything runs, so those that do not fit must queue
    jobs = []
    for t in spec["tasks"]:
        b = bufs[t.task_id]
        if t.kind == "jacobi":
            n, it = t.params["n"], t.params["iters"]
            mem, grid, block = mgb.probe_of(mgb.mgb_jacobi_probe, n, it)
            fn = (lambda b, n, it: lambda st: mgb.mgb_jacobi_enqueue(st, P(b[0]), P(b[1]), n, it))(b, n, it)
        else:
            n = t.params["n"]
            mem, grid, block = mgb.probe_of(mgb.mgb_gemm_f32_probe, n, n, n)
            fn = (lambda b, n: lambda st: mgb.mgb_gemm_f32_enqueue(st, P(b[0]), P(b[1]), P(b[2]), n, n, n))(b, n)
        rc, pl = s.probe(t.task_id, mem, grid, block)
        assert rc in (mgb.MGB_OK, mgb.MGB_WAIT)
        jobs.append((t, rc, pl, fn))
    assert s.stats().n_waiting > 0

    def worker(t, rc, pl, fn):
        try:
            if rc == mgb.MGB_WAIT:
                rc, pl = s.wait(pl.ticket)
            assert rc == mgb.MGB_OK
            assert s.launch(pl.ticket, fn) == 0
            assert s.sync(pl.ticket)[0] == 0
            assert s.complete(pl.ticket) == 0
        except Exception as e:  # noqa: BLE001
            errors.append((t.task_id, e))

    threads = [threading.Thread(target=worker, args=j) for j in jobs]
    for th in threads:
        th.start()
    for th in threads:
        th.join(timeout=100)
    assert not errors, errors
    trace = s.trace()
    dec = assert_trace_matches_replay(s.desc, trace)
    assert (dec["kind"] == oracle.D_WAIT).sum() > 0                    # admission did queue
    # the ledger never exceeded the cap, and every waiter was admitted at some release
    assert trace["free_bytes"].max() <= spec["cap_bytes"]
    admits = trace[trace["kind"] == mgb.MGB_EV_ADMIT]
    assert len(admits) == 32
    # worst waiting time, counted in events between a task's probe and its admission, agrees
    # between the library's log and the replayed schedule (they are the same sequence)
    probe_seq = {int(r["task_id"]): int(r["seq"]) for r in trace if r["kind"] == mgb.MGB_EV_PROBE}
    waits_lib = {int(r["task_id"]): int(r["cause_seq"]) - probe_seq[int(r["task_id"])] for r in admits}
    assert max(waits_lib.values()) > 0
    assert s.destroy() == 0


def _loop_operand(b, lane, e):
    h = (lane.astype(np.uint64) * 2654435761 + b * 40503 + e * 9973 + 12345) & 0xFFFFFFFF
    h ^= h >> 15
    h = (h * 0x2C1B3C6D) & 0xFFFFFFFF
    h ^= h >> 12
    return ((h >> 8).astype(np.float64) / 8388608.0 - 1.0).astype(np.float32)


@pytest.mark.parametrize("bf16", [0, 1])
def test_mfma_loop_diagnostic_sums_what_its_operands_give(bf16):
    # block b multiplies the 32 x depth matrix A_b by its own transpose `iters` times; lane l holds row
    # l % 32 and the depth indices of half l / 32 (one fp32 value, or eight bf16 values), all values a
    # fixed hash of (b, l, element).  A wave's 64 stored floats add up to every entry of all 16 products.
    n_blocks, iters, depth = 8, 5, (16 if bf16 else 2)
    per_lane = depth // 2
    out = torch.zeros(n_blocks * 256, dtype=torch.float32, device=DEV)
    fl = C.c_double(0.0)
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    assert mgb.mgb_mfma_loop_enqueue(st, bf16, n_blocks, iters, P(out), C.byref(fl)) == 0
    torch.cuda.synchronize()
    assert fl.value == n_blocks * 4 * iters * 16 * 2 * 32 * 32 * depth
    want = mag = 0.0
    rows = np.arange(32)
    for b in range(16):
        a = np.empty((32, depth), dtype=np.float32)
        for k in range(depth):
            a[:, k] = _loop_operand(b, rows + 32 * (k // per_lane), k % per_lane)
        if bf16:
            a = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
        a = a.astype(np.float64)
        want += iters * (a @ a.T).sum()
        mag += iters * (np.abs(a) @ np.abs(a).T).sum()
    got = out.cpu().numpy().astype(np.float64).reshape(n_blocks * 4, 64).sum(axis=1)
    assert np.abs(got - want).max() <= 1e-5 * mag
    assert mgb.mgb_mfma_loop_enqueue(st, bf16, 0, iters, P(out), None) == mgb.MGB_E_INVAL
    assert mgb.mgb_mfma_loop_enqueue(st, bf16, n_blocks, 0, P(out), None) == mgb.MGB_E_INVAL
    assert mgb.mgb_mfma_loop_enqueue(st, bf16, n_blocks, iters, None, None) == mgb.MGB_E_INVAL


def test_fetch_and_lds_rate_diagnostics():
    # the two rate probes behind the tile shapes of the MFMA kernels: argument checks, the byte counts
    # they report, and the two orderings the kernels rely on (whole cache lines beat half lines out of
    # L2; swizzled fragment reads beat reads that pile onto the same banks)
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    src = torch.zeros(4 << 20, dtype=torch.uint8, device=DEV)
    sink = torch.zeros(1, dtype=torch.int32, device=DEV)
    nb = C.c_double(0.0)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(fn):
        assert fn() == 0, mgb.mgb_last_error()
        e0.record()
        assert fn() == 0
        e1.record()
        torch.cuda.synchronize()
        return nb.value / e0.elapsed_time(e1)

    fetch = lambda row: mgb.mgb_fetch_rate_enqueue(st, P(src), 2 << 20, row, 8192, 512, 200, P(sink), C.byref(nb))
    half, whole = timed(lambda: fetch(64)), timed(lambda: fetch(128))
    assert nb.value == 512 * 4 * 200 * 8 * 1024
    assert whole > 1.4 * half
    timed(lambda: fetch(1024))
    lds = lambda swz: mgb.mgb_lds_read_rate_enqueue(st, swz, 512, 500, P(sink), C.byref(nb))
    good, bad = timed(lambda: lds(1)), timed(lambda: lds(0))
    assert nb.value == 512 * 256 * 500 * 8 * 16
    assert good > 2 * bad
    assert int(sink.item()) == 0
    inval = mgb.MGB_E_INVAL
    assert mgb.mgb_fetch_rate_enqueue(st, P(src), 2 << 20, 96, 8192, 512, 10, P(sink), None) == inval      # row size
    assert mgb.mgb_fetch_rate_enqueue(st, P(src), 2 << 20, 64, 40, 512, 10, P(sink), None) == inval        # pitch below the row
    assert mgb.mgb_fetch_rate_enqueue(st, P(src), 1024, 128, 8192, 512, 10, P(sink), None) == inval        # footprint below one instruction's span
    assert mgb.mgb_fetch_rate_enqueue(st, None, 2 << 20, 64, 8192, 512, 10, P(sink), None) == inval
    assert mgb.mgb_fetch_rate_enqueue(st, P(src), 2 << 20, 64, 8192, 0, 10, P(sink), None) == inval
    assert mgb.mgb_lds_read_rate_enqueue(st, 1, 512, 0, P(sink), None) == inval
    assert mgb.mgb_lds_read_rate_enqueue(st, 1, 512, 10, None, None) == inval
