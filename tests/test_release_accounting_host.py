"""Host tests (null backend, no GPU) of the stream-ordered release and of the accounting calls.

mgb_task_complete_on_stream credits the ledger when a task's last kernel is enqueued; the tasks
that take over its granules or its bytes must start behind it on the device.  The cases below are
worked by hand; the trace of every case must replay through the independent checker unchanged
(the release is an ordinary COMPLETE to the policy)."""
import ctypes as C

import pytest

import paper_2107_08538_amd as mgb
from helpers import assert_trace_matches_replay, check_ledger_invariants

ONE = (64, 1, 1)


def sched(**kw):
    kw.setdefault("backend", mgb.MGB_BACKEND_NULL)
    return mgb.Sched(**kw)


def grid_for(granules):
    # one-wave workgroups at one workgroup per CU: 32 CUs per granule
    return (32 * granules, 1, 1)


def admit(s, tid, granules, mem=1 << 20):
    rc, pl = s.probe(tid, mem, grid_for(granules), ONE, 1)
    return rc, pl


def launch(s, ticket):
    assert s.launch(ticket, lambda st: 0) == 0


def test_successors_start_behind_the_task_whose_granules_they_take():
    s = sched()
    rc, a = admit(s, 1, 8)
    assert rc == mgb.MGB_OK and a.granule_mask == 0xff and s.deps(a.ticket) == []
    rc, b = admit(s, 2, 4)
    rc2, c = admit(s, 3, 4)
    assert rc == rc2 == mgb.MGB_WAIT
    launch(s, a.ticket)
    assert s.complete_on_stream(a.ticket) == 0          # A's kernels "still run"
    rc, b = s.wait(b.ticket, 0)
    rc2, c = s.wait(c.ticket, 0)
    assert rc == rc2 == mgb.MGB_OK
    assert (b.granule_mask, c.granule_mask) == (0x0f, 0xf0)
    assert s.deps(b.ticket) == [a.ticket] and s.deps(c.ticket) == [a.ticket]
    rc, d = admit(s, 4, 2)
    assert rc == mgb.MGB_WAIT
    launch(s, b.ticket)
    assert s.complete_on_stream(b.ticket) == 0
    rc, d = s.wait(d.ticket, 0)
    assert rc == mgb.MGB_OK and d.granule_mask == 0x03
    assert s.deps(d.ticket) == [b.ticket]               # not A: B already waits for A
    assert s.sync(a.ticket)[0] == 0                     # A is seen finished and forgotten
    assert s.sync(a.ticket)[0] == mgb.MGB_E_UNKNOWN_TICKET
    launch(s, c.ticket)
    assert s.complete(c.ticket) == 0                    # host-observed release: nothing pending on 4..7
    rc, e = admit(s, 5, 2)
    assert rc == mgb.MGB_OK and e.granule_mask == 0x0c and s.deps(e.ticket) == [b.ticket]
    assert s.sync(b.ticket)[0] == 0
    rc, f = admit(s, 6, 4)
    assert rc == mgb.MGB_OK and f.granule_mask == 0xf0 and s.deps(f.ticket) == []
    rc, g = admit(s, 7, 1)
    assert rc == mgb.MGB_WAIT                           # granules 0..3 are D and E, 4..7 is F
    for t in (d, e, f):
        assert s.complete(t.ticket) == 0
    rc, g = s.wait(g.ticket, 0)
    assert rc == mgb.MGB_OK and s.deps(g.ticket) == []  # B retired before G was admitted
    assert s.complete(g.ticket) == 0
    tr = s.trace()
    assert_trace_matches_replay(s.desc, tr)
    check_ledger_invariants(s.desc, tr)
    assert s.destroy() == 0


def test_a_released_ticket_is_gone_for_every_call_but_sync_and_replays_as_unknown():
    s = sched()
    rc, a = admit(s, 1, 8)
    launch(s, a.ticket)
    assert s.complete_on_stream(a.ticket) == 0
    assert s.complete_on_stream(a.ticket) == mgb.MGB_E_UNKNOWN_TICKET
    assert s.complete(a.ticket) == mgb.MGB_E_UNKNOWN_TICKET
    assert s.cancel(a.ticket) == mgb.MGB_E_UNKNOWN_TICKET
    assert s.grow(a.ticket, 1) == mgb.MGB_E_UNKNOWN_TICKET
    assert s.launch(a.ticket, lambda st: 0) == mgb.MGB_E_BAD_STATE
    st = s.stats()
    assert st.n_running == 0 and st.free_granules == 0xff and st.free_bytes == s.desc.mem_cap_bytes
    assert_trace_matches_replay(s.desc, s.trace())
    assert s.destroy() == 0                             # a draining task nobody waited for does not block destroy
    s = sched()
    rc, a = admit(s, 1, 8)
    rc, b = admit(s, 2, 8)
    assert s.complete_on_stream(b.ticket) == mgb.MGB_E_BAD_STATE      # queued, not resident
    assert s.destroy() == mgb.MGB_E_BUSY
    assert s.complete(a.ticket) == 0 and s.wait(b.ticket, 0)[0] == 0 and s.complete(b.ticket) == 0
    assert_trace_matches_replay(s.desc, s.trace())
    assert s.destroy() == 0


def test_bytes_that_may_still_be_in_use_order_the_start_of_whoever_needs_them():
    # SOFT: compute never orders anything, so every dependency below is a memory one
    s = sched(policy=mgb.MGB_POLICY_SOFT, mem_cap_bytes=100)
    rc, x = admit(s, 1, 1, mem=60)
    rc2, y = admit(s, 2, 1, mem=60)
    assert (rc, rc2) == (mgb.MGB_OK, mgb.MGB_WAIT)
    rc, small = admit(s, 3, 1, mem=10)                  # fits beside X: uses no bytes X holds
    assert rc == mgb.MGB_OK and s.deps(small.ticket) == []
    assert s.complete(small.ticket) == 0
    launch(s, x.ticket)
    assert s.complete_on_stream(x.ticket) == 0
    rc, y = s.wait(y.ticket, 0)
    assert rc == mgb.MGB_OK and s.deps(y.ticket) == [x.ticket]       # 60 > 100 - 60 certainly unused
    rc, z = admit(s, 4, 1, mem=30)                      # ledger: 40 free; device: X + Y already hold 120
    assert rc == mgb.MGB_OK and s.deps(z.ticket) == [x.ticket]
    assert s.sync(x.ticket)[0] == 0
    rc, w = admit(s, 5, 1, mem=10)
    assert rc == mgb.MGB_OK and s.deps(w.ticket) == []
    for t in (y, z, w):
        assert s.complete(t.ticket) == 0
    assert_trace_matches_replay(s.desc, s.trace())
    assert s.destroy() == 0


def test_whole_device_policy_chains_every_task_behind_its_predecessor():
    s = sched(policy=mgb.MGB_POLICY_SERIAL, queue_mode=mgb.MGB_QUEUE_FIFO)
    pls = [admit(s, i, 1) for i in range(5)]
    assert [rc for rc, _ in pls] == [mgb.MGB_OK] + [mgb.MGB_WAIT] * 4
    prev = pls[0][1]
    for i in range(1, 5):
        launch(s, prev.ticket)
        assert s.complete_on_stream(prev.ticket) == 0
        rc, cur = s.wait(pls[i][1].ticket, 0)
        assert rc == mgb.MGB_OK and cur.granule_mask == 0xff and s.deps(cur.ticket) == [prev.ticket]
        prev = cur
    assert s.complete(prev.ticket) == 0
    assert_trace_matches_replay(s.desc, s.trace())
    assert s.destroy() == 0


def test_records_follow_a_task_from_probe_to_end():
    s = sched(mem_cap_bytes=100)
    rc, a = admit(s, 11, 8, mem=70)
    rc, b = admit(s, 12, 8, mem=70)
    rc, c = admit(s, 13, 8, mem=70)
    assert s.cancel(c.ticket) == 0
    launch(s, a.ticket)
    assert s.sync(a.ticket)[0] == 0 and s.complete(a.ticket) == 0
    rc, b = s.wait(b.ticket, 0)
    launch(s, b.ticket)
    assert s.complete_on_stream(b.ticket) == 0
    recs, n = s.records()
    assert n == 3 and [recs[i].task_id for i in range(3)] == [11, 12, 13]
    ra, rb, rc_ = recs[0], recs[1], recs[2]
    assert ra.status == mgb.MGB_OK and ra.probe_ns <= ra.admit_ns <= ra.done_ns <= ra.release_ns
    assert ra.granule_mask == 0xff and ra.demand == 8 and ra.mem_bytes == 70
    assert rb.status == mgb.MGB_OK and rb.admit_ns >= ra.release_ns and rb.done_ns == 0   # not seen finished yet
    assert rc_.status == mgb.MGB_TIMEOUT and rc_.admit_ns == 0
    assert s.sync(b.ticket)[0] == 0
    recs, n = s.records(2)
    assert n == 2 and recs[0].ticket == 2 and recs[0].done_ns >= recs[0].release_ns
    assert s.destroy() == 0


def _rec(arr_ms, probe_ms, admit_ms, done_ms, gpu_ms, status=mgb.MGB_OK):
    r = mgb.mgb_task_record()
    r.probe_ns, r.admit_ns, r.done_ns = int(probe_ms * 1e6), int(admit_ms * 1e6), int(done_ms * 1e6)
    r.release_ns = r.done_ns
    r.gpu_ms = gpu_ms
    r.status = status
    return r, int(arr_ms * 1e6)


def test_accounting_on_a_hand_written_set_of_records():
    # Sec. V-A: turnaround = completion - arrival in the queue; throughput over the whole run;
    # kernel slowdown = time when sharing over time on a dedicated device, minus one.
    rows = [_rec(0.0, 0.0, 0.5, 5.0, 1.1), _rec(1.0, 1.5, 1.5, 4.0, 2.0), _rec(2.0, 2.0, 6.0, 10.0, 0.9),
            _rec(3.0, 3.0, 3.0, 3.0, 0.0, mgb.MGB_E_OOM), _rec(0.0, 4.0, 0.0, 0.0, 0.0, mgb.MGB_WAIT)]
    recs = (mgb.mgb_task_record * len(rows))(*[r for r, _ in rows])
    arr = (C.c_uint64 * len(rows))(*[a for _, a in rows])
    ref = (C.c_double * len(rows))(1.0, 2.0, 1.0, 0.0, 0.0)
    out = mgb.mgb_summary()
    assert mgb.mgb_accounting(recs, len(rows), arr, ref, C.byref(out)) == 0
    assert (out.n_done, out.n_crashed, out.n_unfinished) == (3, 1, 1)
    assert out.makespan_ms == pytest.approx(10.0) and out.tasks_per_s == pytest.approx(300.0)
    assert out.mean_turnaround_ms == pytest.approx((5.0 + 3.0 + 8.0) / 3) and out.max_turnaround_ms == pytest.approx(8.0)
    assert out.mean_wait_ms == pytest.approx((0.5 + 0.0 + 4.0) / 3) and out.max_wait_ms == pytest.approx(4.0)
    assert out.gpu_busy_ms == pytest.approx(4.0)
    assert out.max_slowdown == pytest.approx(0.1) and out.mean_slowdown == pytest.approx(0.0, abs=1e-12)
    # without arrival times the probe time stands in: task 2 then turns round in 2.5 ms
    assert mgb.mgb_accounting(recs, 3, None, None, C.byref(out)) == 0
    assert out.mean_turnaround_ms == pytest.approx((5.0 + 2.5 + 8.0) / 3) and out.max_slowdown == 0.0
    # a record that ends before it arrives is refused
    bad, _ = _rec(0.0, 5.0, 5.0, 4.0, 1.0)
    assert mgb.mgb_accounting((mgb.mgb_task_record * 1)(bad), 1, None, None, C.byref(out)) == mgb.MGB_E_INVAL
    assert mgb.mgb_accounting(None, 0, None, None, C.byref(out)) == 0 and out.n_done == 0


# ------------------------------------------------------------------ worker pool (null backend)
def _custom_jobs(n, mems, granules, arrivals_ns=None):
    calls = []

    def body(stream, user):
        calls.append(int(user or 0))
        return 0
    cb = mgb.ENQUEUE_FN(body)
    descs = (mgb.mgb_task_desc * n)()
    for i in range(n):
        d = descs[i]
        d.kind, d.task_id, d.count = mgb.MGB_TASK_CUSTOM, 100 + i, mems[i]
        d.arrival_ns = arrivals_ns[i] if arrivals_ns else 0
        d.ptr[0] = C.cast(cb, C.c_void_p).value
        d.ptr[1] = i + 1
        d.dim[0], d.dim[1], d.dim[2] = 32 * granules[i], 64, 1
    return descs, calls, cb


@pytest.mark.parametrize("flags", [0, mgb.MGB_POOL_RELEASE_ON_STREAM])
@pytest.mark.parametrize("policy", [mgb.MGB_POLICY_HARD, mgb.MGB_POLICY_SOFT, mgb.MGB_POLICY_SERIAL])
def test_pool_runs_a_batch_queue_to_its_end_and_the_trace_replays(policy, flags):
    n = 40
    mems = [10 + (7 * i) % 50 for i in range(n)]
    gran = [1 << (i % 4) for i in range(n)]
    descs, calls, cb = _custom_jobs(n, mems, gran)
    s = sched(policy=policy, mem_cap_bytes=100, max_running=0)
    res = (mgb.mgb_pool_result * n)()
    start = C.c_uint64(0)
    assert mgb.mgb_pool_run(s.h, descs, n, 64, flags, res, C.byref(start)) == 0
    assert sorted(calls) == list(range(1, n + 1))                   # every job's kernels enqueued once
    tr = s.trace()
    dec = assert_trace_matches_replay(s.desc, tr)
    check_ledger_invariants(s.desc, tr)
    # a worker per job and all jobs queued at the start: the probes went out in the order given
    probes = [int(r["task_id"]) for r in tr if r["kind"] == mgb.MGB_EV_PROBE]
    assert probes == [100 + i for i in range(n)]
    for i in range(n):
        r = res[i]
        assert r.status == 0 and r.record.task_id == 100 + i and r.record.status == mgb.MGB_OK
        assert r.arrival_ns == start.value <= r.record.probe_ns <= r.record.admit_ns <= r.record.done_ns
        assert r.record.mem_bytes == mems[i]
    st = s.stats()
    assert st.n_running == 0 and st.n_waiting == 0 and st.free_bytes == 100
    assert s.destroy() == 0


def test_pool_with_arrivals_and_fewer_workers_than_jobs():
    n = 12
    arr = [int(2e6 * (i // 2)) for i in range(n)]                   # two jobs every 2 ms
    arr[3], arr[8] = arr[8], arr[3]                                 # not given in arrival order
    descs, calls, cb = _custom_jobs(n, [1] * n, [8] * n, arr)
    s = sched()
    res = (mgb.mgb_pool_result * n)()
    start = C.c_uint64(0)
    assert mgb.mgb_pool_run(s.h, descs, n, 3, mgb.MGB_POOL_ARRIVALS, res, C.byref(start)) == 0
    assert len(calls) == n
    for i in range(n):
        assert res[i].arrival_ns == start.value + arr[i]
        assert res[i].record.probe_ns >= res[i].arrival_ns          # no job is probed before it arrives
        assert res[i].record.probe_ns - res[i].arrival_ns < 50e6
    # jobs are taken in arrival order
    tr = s.trace()
    probes = [int(r["task_id"]) - 100 for r in tr if r["kind"] == mgb.MGB_EV_PROBE]
    assert [arr[i] for i in probes] == sorted(arr)
    assert_trace_matches_replay(s.desc, tr)
    assert s.destroy() == 0


def test_pool_counts_jobs_lost_to_memory_blind_packing_and_refuses_bad_descriptors():
    n = 6
    descs, calls, cb = _custom_jobs(n, [60] * n, [1] * n)
    s = sched(policy=mgb.MGB_POLICY_CG, mem_cap_bytes=100, max_running=6)
    res = (mgb.mgb_pool_result * n)()
    assert mgb.mgb_pool_run(s.h, descs, n, n, 0, res, None) == 0    # lost jobs are not an error of the run
    lost = [i for i in range(n) if res[i].status == mgb.MGB_E_OOM]
    assert 0 < len(lost) < n and len(calls) == n - len(lost)
    assert all(res[i].record.status == mgb.MGB_E_OOM for i in lost)
    assert_trace_matches_replay(s.desc, s.trace())
    descs[2].kind = 99
    assert mgb.mgb_pool_run(s.h, descs, n, n, 0, res, None) == mgb.MGB_E_INVAL
    assert mgb.mgb_pool_run(s.h, descs, n, 0, 0, res, None) == mgb.MGB_E_INVAL
    assert mgb.mgb_pool_run(s.h, None, 0, 1, 0, None, None) == 0
    assert s.destroy() == 0


def test_growth_into_bytes_that_may_still_be_in_use_and_one_waiter_per_draining_task():
    s = sched(policy=mgb.MGB_POLICY_SOFT, mem_cap_bytes=100)
    rc, x = admit(s, 1, 1, mem=60)
    rc, t = admit(s, 2, 1, mem=20)
    assert s.deps(t.ticket) == []
    launch(s, x.ticket)
    assert s.complete_on_stream(x.ticket) == 0                      # ledger: 80 free, of which 60 may still be in use
    assert s.grow(t.ticket, 20) == mgb.MGB_OK and s.deps(t.ticket) == []            # 20 <= 80 - 60 certainly unused
    assert s.grow(t.ticket, 30) == mgb.MGB_OK and s.deps(t.ticket) == [x.ticket]    # 30 > 60 - 60
    assert s.grow(t.ticket, 40) == mgb.MGB_E_BUSY                   # only 30 left in the ledger
    # two threads may not both wait for the draining task: the second is refused while the first waits
    # (null backend: the wait returns at once, so the calls follow each other and the second finds it gone)
    assert s.sync(x.ticket)[0] == 0 and s.sync(x.ticket)[0] == mgb.MGB_E_UNKNOWN_TICKET
    assert s.complete(t.ticket) == 0
    assert_trace_matches_replay(s.desc, s.trace())
    assert s.destroy() == 0
