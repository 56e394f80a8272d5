"""Host-side checks that run without a GPU: the library loads and exports what the header
declares, and the scheduler core (null backend) agrees with the independent replay."""
import ctypes as C
import os
import re
import threading
import time

import numpy as np
import pytest

import oracle
import paper_2107_08538_amd as mgb
from helpers import assert_trace_matches_replay

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "mgb.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(mgb_[a-z0-9_]+)\s*\(", hdr))
    assert len(declared) >= 29
    for name in declared:
        assert hasattr(mgb.lib, name), name
    assert declared == set(mgb.EXPORTS)


def test_struct_layouts_match_header():
    assert C.sizeof(mgb.mgb_device_desc) == 48
    assert C.sizeof(mgb.mgb_placement) == 56
    assert mgb.TRACE_DT.itemsize == 128
    d = mgb.default_desc()
    assert (d.mem_cap_bytes, d.n_cu, d.granule_cus, d.wave_size) == (288 * 10 ** 9, 256, 32, 64)
    assert (d.max_waves_per_cu, d.max_wg_per_cu, d.policy, d.queue_mode) == (32, 32, 0, 0)


def _null(**kw):
    kw.setdefault("granule_cus", 8)      # 32 granules: the finest partition the checker models
    return mgb.Sched(backend=mgb.MGB_BACKEND_NULL, **kw)


def test_create_rejects_bad_descriptors():
    h = C.c_void_p()
    for kw in (dict(n_cu=0), dict(granule_cus=0), dict(n_cu=250), dict(granule_cus=4),
               dict(policy=9), dict(queue_mode=5), dict(wave_size=0), dict(backend=7)):
        d = mgb.default_desc(backend=mgb.MGB_BACKEND_NULL)
        for k, v in kw.items():
            setattr(d, k, v)
        assert mgb.mgb_sched_create(C.byref(d), C.byref(h)) == mgb.MGB_E_INVAL, kw
    assert mgb.mgb_sched_create(None, C.byref(h)) == mgb.MGB_E_INVAL
    # the HIP backend refuses granules that could leave an XCD without CUs
    d = mgb.default_desc(granule_cus=4)
    assert mgb.mgb_sched_create(C.byref(d), C.byref(h)) == mgb.MGB_E_INVAL


def test_error_paths_leave_the_ledger_unchanged():
    s = _null(mem_cap_bytes=1000)
    rc, pl = s.probe(1, 1001, (1, 1, 1), (64, 1, 1))
    assert rc == mgb.MGB_E_TOO_BIG and s.stats().n_waiting == 0      # never queued
    assert s.probe(1, 10, (0, 1, 1), (64, 1, 1))[0] == mgb.MGB_E_INVAL
    assert s.probe(1, 10, (1, 1, 1), (1025, 1, 1))[0] == mgb.MGB_E_INVAL
    assert s.probe(1, 10, (1, 1, 1), (32, 33, 1))[0] == mgb.MGB_E_INVAL
    assert s.complete(77) == mgb.MGB_E_UNKNOWN_TICKET
    rc, pl = s.probe(2, 600, (1, 1, 1), (64, 1, 1))
    assert rc == mgb.MGB_OK and pl.granule_mask == 1 and pl.stream is None
    rc, pl2 = s.probe(3, 600, (1, 1, 1), (64, 1, 1))
    assert rc == mgb.MGB_WAIT
    assert s.complete(pl2.ticket) == mgb.MGB_E_BAD_STATE              # still waiting
    assert s.cancel(pl.ticket) == mgb.MGB_E_BAD_STATE                 # already running
    assert s.wait(pl2.ticket, 1_000_000)[0] == mgb.MGB_TIMEOUT
    assert s.destroy() == mgb.MGB_E_BUSY
    st = s.stats()
    assert (st.free_bytes, st.n_running, st.n_waiting) == (400, 1, 1)
    assert s.complete(pl.ticket) == mgb.MGB_OK
    assert s.complete(pl.ticket) == mgb.MGB_E_UNKNOWN_TICKET          # double complete
    rc, pl3 = s.wait(pl2.ticket, 0)
    assert rc == mgb.MGB_OK and pl3.ticket == pl2.ticket and pl3.granule_mask == 1
    assert s.complete(pl2.ticket) == mgb.MGB_OK
    assert s.stats().free_bytes == 1000 and s.stats().free_granules == 0xFFFFFFFF
    assert_trace_matches_replay(s.desc, s.trace())
    assert s.destroy() == mgb.MGB_OK


def test_stuck_task_does_not_block_tasks_that_fit():
    s = _null(mem_cap_bytes=1000)
    rc, big = s.probe(1, 900, (100000, 1, 1), (256, 1, 1))            # whole device, never completes
    assert rc == mgb.MGB_OK and big.granule_mask == 0xFFFFFFFF
    rc, w = s.probe(2, 50, (1, 1, 1), (64, 1, 1))
    assert rc == mgb.MGB_WAIT                                         # compute is hard: must wait
    s2 = _null(mem_cap_bytes=1000, max_running=0)
    rc, half = s2.probe(1, 900, (1024, 1, 1), (256, 1, 1))            # half the device, never completes
    assert rc == mgb.MGB_OK and half.granule_mask == 0x0000FFFF
    for i in range(16):
        rc, pl = s2.probe(10 + i, 5, (8, 1, 1), (256, 1, 1))
        assert rc == mgb.MGB_OK and pl.granule_mask == 1 << (16 + i)
        assert list(pl.cu_mask) == [0] * (4 + i // 4) + [0xFF << (8 * (i % 4))] + [0] * (3 - i // 4)


def test_pressure32_footprints_under_both_caps_worked_by_hand():
    """The 32-task memory-pressure mix at its stated footprints (16 x 12 GiB GEMM, 16 x 2 GiB Jacobi,
    alternating, all probing at t = 0), memory as the only hard resource (SOFT, no limit on resident
    tasks).  Cap = summed footprints / 1.5 = 149.33 GiB: ten GEMM + Jacobi pairs make 140 GiB, the
    eleventh GEMM (task 20) would make 152 and waits, the Jacobi tasks 21, 23, 25, 27 still fit
    (142, 144, 146, 148 GiB), task 29 would make 150 and waits, as do all later GEMMs: 24 resident,
    8 queued.  Under the device's full 288e9 bytes (268.2 GiB >= 224) nobody waits for memory."""
    import workloads as W
    GIB = 1 << 30
    spec = W.pressure32()
    assert spec["cap_bytes"] == int(224 * GIB / 1.5)
    for cap, waiting in ((spec["cap_bytes"], [20, 22, 24, 26, 28, 29, 30, 31]), (288 * 10 ** 9, [])):
        s = _null(mem_cap_bytes=cap, policy=mgb.MGB_POLICY_SOFT, max_running=0)
        tickets, queued = {}, []
        for t in spec["tasks"]:
            if t.kind == "gemm_f32":
                mem, grid, block = mgb.probe_of(mgb.mgb_gemm_f32_probe, t.params["m"], t.params["n"], t.params["k"])
                assert mem == 12 * GIB
            else:
                mem, grid, block = mgb.probe_of(mgb.mgb_jacobi_probe, t.params["n"], t.params["iters"])
                assert mem == 2 * GIB
            rc, pl = s.probe(t.task_id, mem, grid, block)
            assert rc in (mgb.MGB_OK, mgb.MGB_WAIT)
            tickets[t.task_id] = pl.ticket
            if rc == mgb.MGB_WAIT:
                queued.append(t.task_id)
        assert queued == waiting
        resident = 32 - len(waiting)
        used = sum((12 if t.task_id % 2 == 0 else 2) * GIB for t in spec["tasks"] if t.task_id not in waiting)
        assert s.stats().free_bytes == cap - used and (not waiting or used == 148 * GIB)
        # the first GEMM to finish lets exactly one waiter in: 12 GiB come back, task 20 (12 GiB) takes them,
        # and nothing is left for task 22 (148 GiB resident again)
        if waiting:
            assert s.complete(tickets[0]) == mgb.MGB_OK
            rc, pl = s.wait(tickets[20], 0)
            assert rc == mgb.MGB_OK
            rc, pl = s.wait(tickets[22], 0)
            assert rc == mgb.MGB_TIMEOUT
            assert s.stats().free_bytes == cap - 148 * GIB
        assert_trace_matches_replay(s.desc, s.trace())
        assert resident == 24 or resident == 32


def test_residency_fact_enters_the_demand_and_the_trace():
    s = _null(mem_cap_bytes=10 ** 6)                                  # 32 granules of 8 CUs
    g, b = (256, 1, 1), (256, 1, 1)                                   # 4 waves per workgroup: 8 per CU by wave slots
    want = {0: 4, 8: 4, 5: 7, 2: 16, 1: 32}                           # 256 / (8 | 8 | 5 | 2 | 1) CUs in granules of 8
    for hint, granules in want.items():
        rc, pl = s.probe(hint, 1, g, b, hint)
        assert rc == mgb.MGB_OK and pl.n_granules == granules, (hint, pl.n_granules)
        assert s.complete(pl.ticket) == mgb.MGB_OK
    tr = s.trace()
    assert [int(r["demand"]) for r in tr if r["kind"] == mgb.MGB_EV_PROBE] == list(want)
    assert_trace_matches_replay(s.desc, tr)
    # the kernels' own facts against the checker's formulas
    lib = oracle.lib()
    lib.orc_gemm_f32_residency.restype = lib.orc_gemm_bf16_residency.restype = lib.orc_conv3x3_residency.restype = C.c_uint64
    U = C.c_uint64
    for m, n, k in ((4096, 4096, 4096), (1024, 1024, 1024), (1000, 3000, 50), (2816, 2816, 64), (1, 8, 32), (129, 257, 17),
                    (2048, 2048, 64)):
        assert mgb.mgb_gemm_f32_residency(m, n, k) == lib.orc_gemm_f32_residency(U(m), U(n), U(k)), (m, n, k)
        assert mgb.mgb_gemm_bf16_residency(m, n, k) == lib.orc_gemm_bf16_residency(U(m), U(n), U(k)), (m, n, k)
    for shp in ((1, 416, 416, 3, 32, 1), (8, 416, 416, 32, 64, 2), (8, 104, 104, 128, 128, 1), (1, 104, 104, 128, 128, 1),
                (2, 416, 416, 3, 64, 1), (1, 5, 6, 5, 7, 1), (8, 208, 208, 64, 64, 1)):
        assert mgb.mgb_conv3x3_residency(*shp) == lib.orc_conv3x3_residency(*[U(x) for x in shp]), shp
    lib.orc_jacobi_residency.restype = C.c_uint64
    for n in (3, 4, 77, 512, 4096, 4097, 65536):
        assert mgb.mgb_jacobi_residency(n) == lib.orc_jacobi_residency(U(n)), n
    assert (mgb.mgb_jacobi_residency(4096), mgb.mgb_jacobi_residency(2048), mgb.mgb_jacobi_residency(2044), mgb.mgb_jacobi_residency(77), mgb.mgb_jacobi_residency(2)) == (2, 2, 3, 8, 0)
    lib.orc_bfs_residency.restype = C.c_uint64
    for n in (1, 1000, 1 << 16, 1 << 18, (1 << 18) + 1, 1 << 19, 1 << 20, (1 << 20) + 1, 1 << 24):
        assert mgb.mgb_bfs_residency(n) == lib.orc_bfs_residency(U(n)), n
    assert (mgb.mgb_bfs_residency(1 << 20), mgb.mgb_bfs_residency(1 << 16), mgb.mgb_bfs_residency(1 << 22)) == (1, 2, 2)
    assert mgb.mgb_gemm_f32_residency(0, 1, 1) == 0


def test_grow_in_the_library():
    s = _null(mem_cap_bytes=1000)
    rc, p1 = s.probe(1, 400, (4, 1, 1), (64, 1, 1))
    rc, p2 = s.probe(2, 700, (4, 1, 1), (64, 1, 1))
    assert rc == mgb.MGB_WAIT
    assert s.grow(p1.ticket, 500) == mgb.MGB_OK and s.stats().free_bytes == 100
    assert s.grow(p1.ticket, 101) == mgb.MGB_E_BUSY and s.stats().free_bytes == 100
    assert s.grow(p2.ticket, 1) == mgb.MGB_E_BAD_STATE
    assert s.grow(99, 1) == mgb.MGB_E_UNKNOWN_TICKET
    assert s.complete(p1.ticket) == mgb.MGB_OK
    rc, pl = s.wait(p2.ticket, 0)
    assert rc == mgb.MGB_OK and s.stats().free_bytes == 300
    assert s.complete(p2.ticket) == mgb.MGB_OK and s.stats().free_bytes == 1000
    assert_trace_matches_replay(s.desc, s.trace())


def test_jacobi_launch_plan_keeps_buffer_parity():
    # the result must end in buffer iters % 2, so the number of (fused) launches has that parity;
    # up to four sweeps per launch below 2048 columns, up to eight from there on
    for n, maxt in ((2044, 4), (1024, 4), (2048, 8), (4096, 8), (16384, 8)):
        for it in list(range(0, 40)) + [50, 100, 127, 128, 129, 1000]:
            c = mgb.mgb_jacobi_launch_count(n, it)
            fewest = (it + maxt - 1) // maxt
            assert c % 2 == it % 2 and fewest <= c <= fewest + (it // 128 + 1), (n, it, c)
    for it in (0, 1, 5, 100):
        assert mgb.mgb_jacobi_launch_count(77, it) == it                 # n % 4 != 0: one sweep per launch
    assert mgb.mgb_jacobi_launch_count(2044, 100) == 26 and mgb.mgb_jacobi_launch_count(2048, 100) == 14 and mgb.mgb_jacobi_launch_count(2, 5) == 0
    assert mgb.mgb_jacobi_launch_count(4096, 100) == 14 and mgb.mgb_jacobi_launch_count(16384, 50) == 8
    assert mgb.mgb_jacobi_launch_count(8192, 8) == 2 and mgb.mgb_jacobi_launch_count(8192, 7) == 1


def test_resident_task_limit():
    assert mgb.default_desc().max_running == 8                        # one per default partition
    s = _null(mem_cap_bytes=10 ** 6, max_running=16)
    pls = [s.probe(i, 1, (8, 1, 1), (256, 1, 1)) for i in range(17)]
    assert [rc for rc, _ in pls] == [mgb.MGB_OK] * 16 + [mgb.MGB_WAIT]
    assert s.stats().free_granules == 0xFFFF0000                      # granules are free, queues are not
    assert s.complete(pls[3][1].ticket) == 0
    rc, pl = s.wait(pls[16][1].ticket, 0)
    assert rc == mgb.MGB_OK and pl.granule_mask == 1 << 3
    assert_trace_matches_replay(s.desc, s.trace())


def test_buddy_blocks_in_the_library():
    s = _null(mem_cap_bytes=10 ** 6, n_cu=64)                         # 8 granules
    wg = lambda g: (64 * g, 1, 1)
    got = []
    for i, g in enumerate((3, 1, 2, 2, 1)):
        rc, pl = s.probe(i, 1, wg(g), (256, 1, 1))
        got.append((rc, pl.granule_mask, pl.n_granules))
    assert got == [(0, 0x0F, 3), (0, 0x10, 1), (0, 0xC0, 2), (1, 0, 2), (0, 0x20, 1)]
    assert_trace_matches_replay(s.desc, s.trace())


def _random_storm(s, rng, n_ops):
    live = []
    for i in range(n_ops):
        if live and rng.random() < 0.1:
            s.grow(live[int(rng.integers(0, len(live)))], int(rng.integers(0, 1500)))   # any outcome is fine
        elif not live or rng.random() < 0.5:
            mem = int(rng.integers(1, 6000))
            grid = (int(rng.integers(0 if rng.random() < 0.02 else 1, 4000)), int(rng.integers(1, 3)), 1)
            block = (int(rng.choice([64, 192, 256, 1024])), 1, 1)
            rc, pl = s.probe(i, mem, grid, block, int(rng.choice([0, 0, 1, 2, 5])))    # with or without a residency fact
            if rc >= 0:
                live.append(pl.ticket)
        else:
            t = live.pop(int(rng.integers(0, len(live))))
            rc = s.complete(t) if rng.random() < 0.85 else s.cancel(t)
            if rc < 0:
                live.append(t)
    for _ in range(len(live) + 1):
        for t in list(live):
            if s.complete(t) == mgb.MGB_OK:
                live.remove(t)
    return live


@pytest.mark.parametrize("policy", [mgb.MGB_POLICY_HARD, mgb.MGB_POLICY_SOFT, mgb.MGB_POLICY_SERIAL])
@pytest.mark.parametrize("mode", [mgb.MGB_QUEUE_BACKFILL, mgb.MGB_QUEUE_FIFO])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_library_decisions_equal_replay_on_random_streams(policy, mode, seed):
    s = _null(mem_cap_bytes=10_000, policy=policy, queue_mode=mode, max_running=[0, 16, 5][seed])
    left = _random_storm(s, np.random.default_rng(seed), 400)
    assert not left
    dec = assert_trace_matches_replay(s.desc, s.trace())
    assert (dec["kind"] == oracle.D_ADMIT).sum() > 20
    assert s.stats().free_bytes == 10_000
    assert s.destroy() == mgb.MGB_OK


def test_cg_policy_equals_replay_and_wakes_the_waiter_of_a_dead_job():
    h = C.c_void_p()
    d = mgb.default_desc(backend=mgb.MGB_BACKEND_NULL, policy=mgb.MGB_POLICY_CG, max_running=0)
    assert mgb.mgb_sched_create(C.byref(d), C.byref(h)) == mgb.MGB_E_INVAL     # CG needs its ratio
    s = _null(mem_cap_bytes=1000, policy=mgb.MGB_POLICY_CG, max_running=2)
    g, b = (4, 1, 1), (64, 1, 1)
    rc, p1 = s.probe(1, 600, g, b)
    assert rc == mgb.MGB_OK and p1.granule_mask == 0xFFFFFFFF
    assert s.probe(2, 600, g, b)[0] == mgb.MGB_E_OOM                           # dies on arrival
    rc, p3 = s.probe(3, 300, g, b)
    assert rc == mgb.MGB_OK
    rc, p4 = s.probe(4, 500, g, b)
    assert rc == mgb.MGB_WAIT
    got = []
    th = threading.Thread(target=lambda: got.append(s.wait(p4.ticket)[0]))
    th.start()
    assert s.complete(p3.ticket) == mgb.MGB_OK                                 # slot opens, 400 < 500
    th.join(10)
    assert got == [mgb.MGB_E_OOM]
    assert s.wait(p4.ticket)[0] == mgb.MGB_E_UNKNOWN_TICKET                    # collected once
    st = s.stats()
    assert (st.n_running, st.n_waiting, st.free_bytes) == (1, 0, 400)
    assert s.complete(p1.ticket) == mgb.MGB_OK
    assert_trace_matches_replay(s.desc, s.trace())
    for seed, mode in ((0, mgb.MGB_QUEUE_BACKFILL), (1, mgb.MGB_QUEUE_FIFO)):
        s = _null(mem_cap_bytes=10_000, policy=mgb.MGB_POLICY_CG, queue_mode=mode, max_running=4)
        _random_storm(s, np.random.default_rng(seed), 400)
        dec = assert_trace_matches_replay(s.desc, s.trace())
        assert ((dec["kind"] == oracle.D_REJECT) & (dec["code"] == mgb.MGB_E_OOM)).sum() > 3
        assert s.stats().free_bytes == 10_000 and s.stats().n_running == 0


def test_a_release_wakes_exactly_the_waiters_it_concerns():
    # every waiter sleeps on a condition variable of its own; two threads on one ticket share the
    # scheduler's; a cancelled ticket's waiter is told; waiters of tasks that still do not fit sleep on
    s = _null(mem_cap_bytes=1000)
    whole, b = (100000, 1, 1), (256, 1, 1)
    rc, p1 = s.probe(1, 100, whole, b)
    assert rc == mgb.MGB_OK
    waits = [s.probe(i, 100, whole, b) for i in (2, 3, 4)]
    assert [rc for rc, _ in waits] == [mgb.MGB_WAIT] * 3
    t2, t3, t4 = (pl.ticket for _, pl in waits)
    got = {}
    def waiter(name, ticket, timeout=-1):
        got[name] = s.wait(ticket, timeout)[0]
    threads = [threading.Thread(target=waiter, args=("a2", t2)), threading.Thread(target=waiter, args=("b2", t2)),
               threading.Thread(target=waiter, args=("a3", t3)), threading.Thread(target=waiter, args=("a4", t4))]
    for th in threads:
        th.start()
    time.sleep(0.05)
    assert s.cancel(t4) == mgb.MGB_OK                     # its waiter returns with "unknown ticket"
    threads[3].join(10)
    assert got == {"a4": mgb.MGB_E_UNKNOWN_TICKET}
    assert s.complete(p1.ticket) == mgb.MGB_OK            # admits task 2 only (whole-device demands)
    threads[0].join(10)
    threads[1].join(10)
    assert got["a2"] == mgb.MGB_OK and got["b2"] == mgb.MGB_OK and "a3" not in got
    assert s.complete(t2) == mgb.MGB_OK
    threads[2].join(10)
    assert got["a3"] == mgb.MGB_OK
    assert s.wait(t3, 1000)[0] == mgb.MGB_OK              # already admitted: returns at once
    assert s.complete(t3) == mgb.MGB_OK and s.destroy() == 0


def test_small_device_and_other_granule_shapes_equal_replay():
    for n_cu, g in ((32, 8), (64, 2), (24, 1), (256, 64)):
        s = _null(mem_cap_bytes=5000, n_cu=n_cu, granule_cus=g, max_wg_per_cu=8, max_waves_per_cu=40)
        _random_storm(s, np.random.default_rng(n_cu), 300)
        assert_trace_matches_replay(s.desc, s.trace())


def test_concurrent_probe_complete_storm_is_consistent():
    s = _null(mem_cap_bytes=50_000)
    errors = []

    def worker(k):
        rng = np.random.default_rng(100 + k)
        try:
            for i in range(150):
                mem = int(rng.integers(1, 20_000))
                grid = (int(rng.integers(1, 3000)), 1, 1)
                rc, pl = s.probe(k * 1000 + i, mem, grid, (256, 1, 1))
                if rc == mgb.MGB_WAIT:
                    rc, pl = s.wait(pl.ticket, -1)
                assert rc == mgb.MGB_OK and pl.granule_mask != 0
                assert s.complete(pl.ticket) == mgb.MGB_OK
        except Exception as e:          # noqa: BLE001
            errors.append(e)

    threads = [threading.Thread(target=worker, args=(k,)) for k in range(8)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=120)
    assert not errors and not any(t.is_alive() for t in threads)
    st = s.stats()
    assert (st.free_bytes, st.n_running, st.n_waiting) == (50_000, 0, 0)
    assert_trace_matches_replay(s.desc, s.trace())       # whatever the interleaving was, it replays
    assert s.destroy() == mgb.MGB_OK


def test_launch_and_sync_with_null_backend_and_trace_dump(tmp_path):
    s = _null()
    rc, pl = s.probe(5, 100, (10, 1, 1), (256, 1, 1))
    seen = []
    assert s.launch(pl.ticket, lambda stream: seen.append(stream) or 0) == 0
    assert seen == [None]
    assert s.launch(pl.ticket, lambda stream: 7) == 7                 # enqueue status is passed back
    assert s.launch(999, lambda stream: 0) == mgb.MGB_E_UNKNOWN_TICKET
    assert s.sync(pl.ticket) == (0, 0.0)
    assert s.complete(pl.ticket) == 0
    p = str(tmp_path / "trace.jsonl")
    assert s.dump(p) == 0
    import json
    lines = [json.loads(l) for l in open(p)]
    assert [l["kind"] for l in lines] == [0, 16, 1, 19] and lines[1]["cu_mask"][0] == 0xFF


def test_probe_functions_agree_with_checker_formulas():
    out = (C.c_uint64 * 7)()
    for n in (3, 4, 5, 64, 77, 512, 1023, 1024, 1025, 4096, 16384):
        mem, grid, block = mgb.probe_of(mgb.mgb_jacobi_probe, n, 10)
        oracle.lib().orc_jacobi_probe(C.c_uint64(n), C.c_uint64(10), out)
        assert [mem, *grid.tuple(), *block.tuple()] == list(out), n
    for n, it in ((8192, 1), (8192, 4), (8192, 5), (8192, 6), (8192, 100), (8188, 50), (16384, 50), (65536, 7), (4096, 6),
                  (4096, 96), (4096, 100), (4096, 8), (4096, 9), (4092, 7), (4100, 200), (2048, 100), (4096, 1000), (4096, 0)):
        mem, grid, block = mgb.probe_of(mgb.mgb_jacobi_probe, n, it)
        oracle.lib().orc_jacobi_probe(C.c_uint64(n), C.c_uint64(it), out)
        assert [mem, *grid.tuple(), *block.tuple()] == list(out), (n, it)
    for m, n, k in ((1, 1, 1), (128, 128, 16), (129, 257, 17), (256, 256, 256), (4096, 4096, 4096),
                    (32768, 32768, 32768), (1000, 3000, 50), (1024, 1024, 1024), (1408, 1536, 64), (1408, 1408, 64),
                    (1000, 3000, 48), (1000, 3002, 48), (2816, 2816, 64), (4096, 4096, 64), (4096, 3840, 64), (8192, 8192, 16),
                    (4544, 4544, 64), (6528, 6528, 16), (7552, 7552, 16), (5504, 5504, 32), (4096, 4100, 32)):
        mem, grid, block = mgb.probe_of(mgb.mgb_gemm_f32_probe, m, n, k)
        oracle.lib().orc_gemm_f32_probe(C.c_uint64(m), C.c_uint64(n), C.c_uint64(k), out)
        assert [mem, *grid.tuple(), *block.tuple()] == list(out), (m, n, k)
    for m, n, k in ((1, 1, 1), (129, 257, 17), (4096, 4096, 4096), (8192, 1024, 64), (300, 520, 64), (300, 520, 48),
                    (300, 524, 64), (1, 8, 32), (2560, 2560, 2560), (2816, 2816, 64), (3072, 2816, 64), (8192, 8192, 8192)):
        mem, grid, block = mgb.probe_of(mgb.mgb_gemm_bf16_probe, m, n, k)
        oracle.lib().orc_gemm_bf16_probe(C.c_uint64(m), C.c_uint64(n), C.c_uint64(k), out)
        assert [mem, *grid.tuple(), *block.tuple()] == list(out), (m, n, k)
    for b, h, w, ci, co, st in ((1, 416, 416, 3, 32, 1), (8, 416, 416, 32, 64, 2), (2, 13, 11, 512, 512, 2),
                                (1, 5, 6, 5, 7, 1), (3, 26, 26, 40, 200, 1), (8, 104, 104, 128, 128, 1),
                                (1, 104, 104, 128, 128, 1), (8, 26, 26, 512, 512, 2), (2, 416, 416, 3, 64, 1),
                                (2, 416, 416, 3, 32, 2), (1, 64, 64, 3, 36, 1), (4, 208, 208, 64, 64, 1),
                                (1, 52, 52, 96, 72, 1), (1, 52, 52, 96, 68, 1)):
        mem, grid, block = mgb.probe_of(mgb.mgb_conv3x3_probe, b, h, w, ci, co, st)
        oracle.lib().orc_conv3x3_probe(*[C.c_uint64(x) for x in (b, h, w, ci, co, st)], out)
        assert [mem, *grid.tuple(), *block.tuple()] == list(out), (b, h, w, ci, co, st)
    import workloads as W
    for b, h in ((1, 416), (8, 416), (2, 104), (1, 17), (4, 208), (3, 64), (2, 416)):
        layers = W.cnn_layers(h, h)
        arr = (mgb.mgb_conv_layer * 10)(*[mgb.mgb_conv_layer(L["c_in"], L["c_out"], L["stride"]) for L in layers])
        mem, act, ob = C.c_uint64(), C.c_uint64(), C.c_uint64()
        g, blk = mgb.mgb_dim3(), mgb.mgb_dim3()
        assert mgb.mgb_cnn_probe(arr, 10, b, h, h, C.byref(mem), C.byref(act), C.byref(ob), C.byref(g), C.byref(blk)) == 0
        flat = (C.c_uint64 * 30)(*[x for L in layers for x in (L["c_in"], L["c_out"], L["stride"])])
        oracle.lib().orc_cnn_probe(flat, C.c_uint64(10), C.c_uint64(b), C.c_uint64(h), C.c_uint64(h), out)
        assert [mem.value, *g.tuple(), *blk.tuple()] == list(out), (b, h)
    for n, m in ((1, 0), (100, 300), (1 << 16, 1 << 19), (1 << 20, 16777208), (1 << 22, 1 << 26), (5000000, 10)):
        mem, grid, block = mgb.probe_of(mgb.mgb_bfs_probe, n, m)
        oracle.lib().orc_bfs_probe(C.c_uint64(n), C.c_uint64(m), out)
        assert [mem, *grid.tuple(), *block.tuple()] == list(out), (n, m)
        # counters + two queues of n entries + three bitmaps of n bits (256-byte pieces), written out
        work = 256 + 2 * (-(-n * 4 // 256) * 256) + 3 * (-(-(-(-n // 32)) // 64) * 64 * 4)
        assert mem == (n + 1 + m) * 4 + n * 4 + work and mgb.mgb_bfs_work_bytes(n) == work
    mem, grid, block = mgb.mgb_dim3(), None, None
    assert mgb.mgb_jacobi_probe(2, 1, C.byref(C.c_uint64()), C.byref(mgb.mgb_dim3()),
                                C.byref(mgb.mgb_dim3())) == mgb.MGB_E_UNSUPPORTED
    assert mgb.mgb_gemm_f32_probe(0, 1, 1, C.byref(C.c_uint64()), C.byref(mgb.mgb_dim3()),
                                  C.byref(mgb.mgb_dim3())) == mgb.MGB_E_UNSUPPORTED


def test_trace_keeps_the_last_million_records():
    # 2^20 records are kept at most; at the cap the older half goes.  A probe + complete pair
    # logs four records (two inputs, two decisions).
    s = _null()
    pairs = (1 << 18) + 1000
    for i in range(pairs):
        rc, pl = s.probe(i, 1, (1, 1, 1), (64, 1, 1))
        assert rc == mgb.MGB_OK
        assert s.complete(pl.ticket) == mgb.MGB_OK
    st = s.stats()
    assert st.n_events == 4 * pairs > (1 << 20)
    tr = s.trace()                                   # reads from seq 0: starts at the oldest record kept
    assert len(tr) == st.n_events - (1 << 19)
    assert np.array_equal(tr["seq"], np.arange(1 << 19, st.n_events, dtype=np.uint64))
    assert tr["kind"][-1] == mgb.MGB_EV_RELEASE
    tail = np.zeros(8, dtype=mgb.TRACE_DT)
    vp = C.c_void_p(tail.ctypes.data)
    assert mgb.mgb_trace_read(s.h, st.n_events - 2, vp, 8) == 2 and tail["seq"][1] == st.n_events - 1
    assert mgb.mgb_trace_read(s.h, st.n_events, vp, 8) == 0
    assert s.destroy() == 0


def test_header_is_plain_c(tmp_path):
    # the boundary is a C ABI: the header must compile as C99 on its own, and the record sizes that
    # cross it must be what the binding assumes
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("gcc not found")
    src = tmp_path / "hdr.c"
    src.write_text('#include "mgb.h"\n'
                   "int a[sizeof(mgb_trace_rec) == 128 ? 1 : -1];\n"
                   "int b[sizeof(mgb_task_record) == %d ? 1 : -1];\n"
                   "int c[sizeof(mgb_pool_result) == %d ? 1 : -1];\n"
                   "int d[sizeof(mgb_task_desc) == %d ? 1 : -1];\n"
                   "int e[sizeof(mgb_summary) == %d ? 1 : -1];\n"
                   "int f[sizeof(mgb_placement) == %d ? 1 : -1];\n"
                   "int main(void) { mgb_task_desc j = {0}; j.kind = MGB_TASK_CUSTOM; return (int)j.kind - 5; }\n"
                   % (C.sizeof(mgb.mgb_task_record), C.sizeof(mgb.mgb_pool_result), C.sizeof(mgb.mgb_task_desc),
                      C.sizeof(mgb.mgb_summary), C.sizeof(mgb.mgb_placement)))
    inc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", inc, "-fsyntax-only", str(src)],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
