"""Lazy runtime (Sec. III-A) without a GPU: the library on the null backend ("device memory" is
host memory) against the plain-Python model -- same copied-back bytes as eager execution, same
probes / growths / completions towards the scheduler, decisions replayed by the checker -- and the
task-construction algorithm's pins."""
import ctypes as C
import threading

import numpy as np
import pytest

import oracle
from oracle.lazy_model import LazyModel, build_gpu_tasks
import paper_2107_08538_amd as mgb
from helpers import assert_trace_matches_replay


def _f32(view, n):
    return view[:4 * n].view(np.float32)


def k_vadd(args, n):
    with np.errstate(all="ignore"):          # random programs feed arbitrary bit patterns
        _f32(args[2], n)[:] = _f32(args[0], n) + _f32(args[1], n)


def k_scale(args, p):
    n, f = p
    with np.errstate(all="ignore"):
        _f32(args[0], n)[:] *= np.float32(f)


def k_acc(args, n):
    with np.errstate(all="ignore"):
        _f32(args[1], n)[:] += _f32(args[0], n)


KERNELS = {"vadd": k_vadd, "scale": k_scale, "acc": k_acc}


def _real_view(ptr, nbytes):
    return np.ctypeslib.as_array((C.c_uint8 * nbytes).from_address(ptr))


class Both:
    """Runs one program through the library (null backend) and through the model."""

    def __init__(self, **sched_kw):
        sched_kw.setdefault("granule_cus", 8)
        self.s = mgb.Sched(backend=mgb.MGB_BACKEND_NULL, **sched_kw)
        self.z = mgb.Lazy(self.s)
        self.m = LazyModel(KERNELS)
        self.p = {}          # name -> (pseudo, model handle, bytes)

    def malloc(self, name, n):
        rc, pseudo = self.z.malloc(n)
        assert rc == 0 and pseudo >> 56 == 0xA5
        self.p[name] = (pseudo, self.m.malloc(n), n)

    def h2d(self, name, off, data):
        buf = np.frombuffer(bytes(data), dtype=np.uint8).copy()
        assert self.z.memcpy_h2d(self.p[name][0] + off, buf.ctypes.data, buf.size) == 0
        buf[:] = 0xEE                                    # the caller may reuse its buffer at once
        self.m.memcpy_h2d(self.p[name][1], off, data)

    def memset(self, name, off, val, n):
        assert self.z.memset(self.p[name][0] + off, val, n) == 0
        self.m.memset(self.p[name][1], off, val, n)

    def launch(self, task_id, kernel, args, grid, block, params, timeout_ns=-1):
        rc, real, pl = self.z.launch_prepare(task_id, [self.p[n][0] + off for n, off in args], grid, block, timeout_ns)
        if rc != 0:
            return rc
        KERNELS[kernel]([_real_view(r, self.p[n][2] - off) for r, (n, off) in zip(real, args)], params)
        self.m.launch(task_id, kernel, [(self.p[n][1], off) for n, off in args], grid, block, params)
        return 0

    def d2h(self, name, off, n):
        out = np.zeros(n, dtype=np.uint8)
        assert self.z.memcpy_d2h(out.ctypes.data, self.p[name][0] + off, n) == 0
        want = self.m.memcpy_d2h(self.p[name][1], off, n)
        assert out.tobytes() == want, name
        return out

    def free(self, name):
        pseudo, h, _ = self.p.pop(name)
        assert self.z.free(pseudo) == 0
        self.m.free(h)

    def check_scheduler_traffic(self):
        """What reached the scheduler, in order, is what the model derives; its decisions replay."""
        tr = self.s.trace()
        got = []
        for r in tr:
            k = int(r["kind"])
            if k == mgb.MGB_EV_PROBE:
                got.append(("probe", int(r["task_id"]), int(r["mem_bytes"]), tuple(int(x) for x in r["grid"]),
                            tuple(int(x) for x in r["block"])))
            elif k == mgb.MGB_EV_GROW:
                got.append(("grow", int(r["ticket"]), int(r["mem_bytes"])))
            elif k == mgb.MGB_EV_COMPLETE:
                got.append(("complete", int(r["ticket"])))
        assert got == self.m.sched_inputs
        if len(tr):
            assert_trace_matches_replay(self.s.desc, tr)


def test_vector_add_task_of_the_paper_is_one_probe_for_three_buffers():
    # the example task of Sec. III-A: three allocations, two copies in, a launch, a copy out, three frees
    n = 1000
    b = Both(mem_cap_bytes=1 << 20)
    a_h = np.arange(n, dtype=np.float32)
    b_h = np.full(n, 0.5, dtype=np.float32)
    for name in ("dA", "dB", "dC"):
        b.malloc(name, 4 * n)
    b.h2d("dA", 0, a_h.tobytes())
    b.h2d("dB", 0, b_h.tobytes())
    st = b.z.stats()
    assert (st.n_objects, st.n_bound, st.n_tasks, st.recorded_ops, st.staged_bytes) == (3, 0, 0, 2, 8 * n)
    assert len(b.s.trace()) == 0 and b.s.stats().free_bytes == 1 << 20     # nothing has reached the scheduler
    assert b.launch(7, "vadd", [("dA", 0), ("dB", 0), ("dC", 0)], (4, 1, 1), (256, 1, 1), n) == 0
    st = b.z.stats()
    assert (st.n_bound, st.n_tasks, st.replayed_ops, st.staged_bytes) == (3, 1, 2, 0)
    assert b.s.stats().free_bytes == (1 << 20) - 12 * n                     # footprint = the three buffers
    out = b.d2h("dC", 0, 4 * n).view(np.float32)
    assert np.array_equal(out, a_h + b_h)
    b.free("dA")
    b.free("dB")
    assert b.s.stats().n_running == 1                                       # the task lives while it owns memory
    b.free("dC")
    assert b.s.stats().n_running == 0 and b.s.stats().free_bytes == 1 << 20
    assert b.m.sched_inputs == [("probe", 7, 12 * n, (4, 1, 1), (256, 1, 1)), ("complete", 1)]
    b.check_scheduler_traffic()
    assert b.z.destroy() == 0


def test_two_kernels_sharing_an_array_are_one_task():
    # k1 writes C, k2 reads it (the paper's example for merging): one task; what the first launch
    # did not name is asked for when the second arrives; in total what Algorithm 1 merges statically
    n = 256
    b = Both(mem_cap_bytes=1 << 20)
    for name in ("A", "B", "C", "D"):
        b.malloc(name, 4 * n)
    b.h2d("A", 0, np.ones(n, np.float32).tobytes())
    b.h2d("B", 0, np.full(n, 2, np.float32).tobytes())
    b.h2d("D", 0, np.full(n, 10, np.float32).tobytes())
    assert b.launch(1, "vadd", [("A", 0), ("B", 0), ("C", 0)], (1, 1, 1), (256, 1, 1), n) == 0
    assert b.launch(1, "acc", [("C", 0), ("D", 0)], (3, 1, 1), (128, 1, 1), n) == 0
    assert np.array_equal(b.d2h("D", 0, 4 * n).view(np.float32), np.full(n, 13, np.float32))
    assert b.m.sched_inputs == [("probe", 1, 12 * n, (1, 1, 1), (256, 1, 1)), ("grow", 1, 4 * n)]
    static = build_gpu_tasks([dict(memobjs="ABC", allocs=dict(A=4 * n, B=4 * n, C=4 * n), grid=(1, 1, 1), block=(256, 1, 1)),
                              dict(memobjs="CD", allocs=dict(C=4 * n, D=4 * n), grid=(3, 1, 1), block=(128, 1, 1))])
    assert len(static) == 1 and static[0]["mem_bytes"] == 16 * n == 12 * n + 4 * n
    assert static[0]["launches"] == [0, 1] and static[0]["grid"] == (3, 1, 1)      # the launch with more waves (6 against 4)
    for name in "ABCD":
        b.free(name)
    b.check_scheduler_traffic()
    assert b.s.stats().free_bytes == 1 << 20 and b.z.destroy() == 0


def test_task_construction_pins():
    g, blk = (1, 1, 1), (64, 1, 1)
    L = lambda objs, **alloc: dict(memobjs=objs, allocs=alloc, grid=g, block=blk)
    # nothing shared: one task per launch, footprint = its own allocations
    t = build_gpu_tasks([L("A", A=10), L("B", B=20), L("C", C=30)])
    assert [(x["launches"], x["mem_bytes"]) for x in t] == [([0], 10), ([1], 20), ([2], 30)]
    # everything shares one object: one task, every allocation counted once
    t = build_gpu_tasks([L("AX", A=10, X=1), L("BX", B=20, X=1), L("CX", C=30, X=1)])
    assert [(x["launches"], x["mem_bytes"]) for x in t] == [([0, 1, 2], 61)]
    # a chain: 0-1 share C, 1-3 share E, 2 is alone; sharing is transitive
    t = build_gpu_tasks([L("ABC", A=40, B=40, C=40), L("CDE", C=40, D=8, E=8), L("F", F=100), L("EG", E=8, G=16)])
    assert [(x["launches"], x["mem_bytes"]) for x in t] == [([0, 1, 3], 152), ([2], 100)]
    # the order of the launches does not change the partition
    t = build_gpu_tasks([L("EG", E=8, G=16), L("F", F=100), L("CDE", C=40, D=8, E=8), L("ABC", A=40, B=40, C=40)])
    assert [(sorted(x["memobjs"]), x["mem_bytes"]) for x in t] == [(list("ABCDEG"), 152), (["F"], 100)]
    # brute force on small random instances: tasks = connected components of "share an object"
    rng = np.random.default_rng(0)
    for _ in range(50):
        n = int(rng.integers(1, 8))
        launches = [L("".join(rng.choice(list("ABCDEFGH"), int(rng.integers(1, 3)), replace=False))) for _ in range(n)]
        for l in launches:
            l["allocs"] = {o: 1 for o in l["memobjs"]}
        comp = list(range(n))
        for _ in range(n):
            for i in range(n):
                for j in range(n):
                    if set(launches[i]["memobjs"]) & set(launches[j]["memobjs"]):
                        comp[i] = comp[j] = min(comp[i], comp[j])
        want = sorted(sorted(i for i in range(n) if comp[i] == c) for c in set(comp))
        assert sorted(x["launches"] for x in build_gpu_tasks(launches)) == want


def test_a_launch_that_touches_two_tasks_fuses_them():
    n = 64
    b = Both(mem_cap_bytes=1 << 20)
    for name in ("A", "B", "C", "D"):
        b.malloc(name, 4 * n)
        b.h2d(name, 0, np.full(n, ord(name) - 64, np.float32).tobytes())
    assert b.launch(1, "scale", [("A", 0)], (1, 1, 1), (64, 1, 1), (n, 2.0)) == 0          # task 1 {A}
    assert b.launch(2, "acc", [("B", 0), ("C", 0)], (1, 1, 1), (64, 1, 1), n) == 0         # task 2 {B, C}
    assert b.z.stats().n_tasks == 2 and b.s.stats().n_running == 2
    assert b.launch(3, "vadd", [("A", 0), ("C", 0), ("D", 0)], (1, 1, 1), (64, 1, 1), n) == 0   # fuses, brings D
    assert b.z.stats().n_tasks == 1 and b.s.stats().n_running == 2                          # both tickets stay resident
    assert np.array_equal(b.d2h("D", 0, 4 * n).view(np.float32), np.full(n, 2 * 1 + (2 + 3), np.float32))
    for name in "ABC":
        b.free(name)
    assert b.s.stats().n_running == 2
    b.free("D")                                                                             # the last object: both tickets complete
    assert b.s.stats().n_running == 0
    assert b.m.sched_inputs == [("probe", 1, 4 * n, (1, 1, 1), (64, 1, 1)), ("probe", 2, 8 * n, (1, 1, 1), (64, 1, 1)),
                                ("grow", 1, 4 * n), ("complete", 1), ("complete", 2)]
    b.check_scheduler_traffic()
    assert b.z.destroy() == 0


def test_recorded_copies_keep_their_bytes_order_and_offsets():
    b = Both(mem_cap_bytes=1 << 16)
    b.malloc("X", 64)
    b.memset("X", 0, 0x11, 64)
    b.h2d("X", 8, bytes(range(16)))
    b.memset("X", 12, 0xFF, 4)                         # later operations overwrite earlier ones
    b.h2d("X", 60, b"\x01\x02\x03\x04")
    want = b.d2h("X", 0, 64).copy()                    # before any launch: served from the recording
    assert want[8] == 0 and want[12] == 0xFF and want[63] == 4 and want[0] == 0x11
    assert b.z.stats().n_bound == 0 and len(b.s.trace()) == 0
    b.malloc("Y", 64)
    assert b.launch(1, "acc", [("X", 32), ("Y", 0)], (1, 1, 1), (64, 1, 1), 4) == 0   # argument with an offset
    assert np.array_equal(b.d2h("X", 0, 64), want)
    b.h2d("X", 0, b"\x7f" * 8)                         # after the launch: straight to the device copy
    assert b.d2h("X", 0, 9).tolist() == [0x7F] * 8 + [0]
    assert b.z.stats().recorded_ops == 4 and b.z.stats().replayed_ops == 4
    b.free("X")
    b.free("Y")
    b.check_scheduler_traffic()
    assert b.z.destroy() == 0


def test_errors_and_admission_limits():
    b = Both(mem_cap_bytes=1000)
    z = b.z
    assert z.malloc(1 << 41)[0] == mgb.MGB_E_TOO_BIG
    assert z.memset(0xA5 << 56 | 77 << 40, 0, 1) == mgb.MGB_E_UNKNOWN_TICKET and z.free(12345) == mgb.MGB_E_UNKNOWN_TICKET
    b.malloc("A", 600)
    b.malloc("B", 600)
    b.malloc("C", 300)
    assert z.memset(b.p["A"][0] + 599, 0, 2) == mgb.MGB_E_INVAL                 # runs past the object
    assert z.free(b.p["A"][0] + 8) == mgb.MGB_E_UNKNOWN_TICKET                  # not a base address
    assert z.destroy() == mgb.MGB_E_BUSY
    rc, real, pl = z.launch_prepare(1, [b.p["A"][0], b.p["B"][0]], (1, 1, 1), (64, 1, 1))
    assert rc == mgb.MGB_E_TOO_BIG and z.stats().n_bound == 0                   # 1200 > cap: never admitted
    assert b.launch(1, "scale", [("A", 0)], (1, 1, 1), (64, 1, 1), (1, 1.0)) == 0
    # B (600) does not fit beside A (600 of 1000): a new task would wait, so give it 1 ms
    assert b.launch(2, "scale", [("B", 0)], (1, 1, 1), (64, 1, 1), (1, 1.0), timeout_ns=1_000_000) == mgb.MGB_TIMEOUT
    assert z.stats().n_bound == 1 and b.s.stats().n_waiting == 0                # the probe was withdrawn
    # growing A's task by B fails without side effects, by C succeeds
    rc, _, _ = z.launch_prepare(1, [b.p["A"][0], b.p["B"][0]], (1, 1, 1), (64, 1, 1))
    assert rc == mgb.MGB_E_BUSY and z.stats().n_bound == 1 and b.s.stats().free_bytes == 400
    assert b.launch(1, "acc", [("A", 0), ("C", 0)], (1, 1, 1), (64, 1, 1), 1) == 0
    assert b.s.stats().free_bytes == 100
    for name in "ABC":
        b.free(name)
    assert b.s.stats().free_bytes == 1000 and z.destroy() == 0
    assert_trace_matches_replay(b.s.desc, b.s.trace())


@pytest.mark.parametrize("seed", range(8))
def test_random_programs_equal_eager_execution(seed):
    rng = np.random.default_rng(seed)
    b = Both(mem_cap_bytes=1 << 22, max_running=0)
    names = []
    for step in range(120):
        r = rng.random()
        if r < 0.22 or len(names) < 3:
            name = "o%d" % step
            b.malloc(name, 4 * int(rng.integers(8, 64)))
            b.memset(name, 0, int(rng.integers(0, 64)), b.p[name][2])    # a program may not read bytes it never wrote
            names.append(name)
        elif r < 0.45:
            name = names[int(rng.integers(len(names)))]
            size = b.p[name][2]
            off = 4 * int(rng.integers(0, size // 4))
            n = int(rng.integers(0, size - off + 1))
            if rng.random() < 0.5:
                b.h2d(name, off, rng.standard_normal(16).astype(np.float32).tobytes()[:n] if n <= 64 else
                      rng.integers(0, 255, n, dtype=np.uint8).tobytes())
            else:
                b.memset(name, off, int(rng.integers(0, 256)), n)
        elif r < 0.75:
            k = ["vadd", "scale", "acc"][int(rng.integers(3))]
            need = {"vadd": 3, "scale": 1, "acc": 2}[k]
            picks = [names[int(i)] for i in rng.choice(len(names), need, replace=len(names) < need)]
            if k != "scale" and len(set(picks)) != len(picks):
                continue
            n = min(b.p[p][2] for p in picks) // 4
            params = (n, float(rng.integers(1, 4))) if k == "scale" else n
            # keep values finite: refill inputs that a long chain of adds has blown up is not needed for 120 steps
            assert b.launch(step, k, [(p, 0) for p in picks], (int(rng.integers(1, 64)), 1, 1), (64, 1, 1), params) == 0
        elif r < 0.9:
            name = names[int(rng.integers(len(names)))]
            b.d2h(name, 0, b.p[name][2])
        else:
            name = names.pop(int(rng.integers(len(names))))
            b.free(name)
    for name in list(names):
        b.d2h(name, 0, b.p[name][2])
        b.free(name)
    st = b.z.stats()
    assert (st.n_objects, st.n_bound, st.n_tasks, st.staged_bytes) == (0, 0, 0, 0)
    assert b.s.stats().n_running == 0 and b.s.stats().free_bytes == 1 << 22
    b.check_scheduler_traffic()
    assert b.z.destroy() == 0


def test_two_clients_contend_for_memory_through_the_scheduler():
    # two programs, each its own lazy instance, on one scheduler whose cap holds only one of them
    s = mgb.Sched(backend=mgb.MGB_BACKEND_NULL, mem_cap_bytes=1000, granule_cus=8)
    results, errors = {}, []

    def program(i):
        try:
            z = mgb.Lazy(s)
            rc, a = z.malloc(800)
            src = np.full(200, float(i), np.float32)
            assert z.memcpy_h2d(a, src.ctypes.data, 800) == 0
            rc, real, pl = z.launch_prepare(i, [a], (1, 1, 1), (64, 1, 1))
            assert rc == 0
            k_scale([_real_view(real[0], 800)], (200, 3.0))
            out = np.zeros(200, np.float32)
            assert z.memcpy_d2h(out.ctypes.data, a, 800) == 0
            results[i] = out
            assert z.free(a) == 0 and z.destroy() == 0
        except Exception as e:   # noqa: BLE001
            errors.append(repr(e))

    th = [threading.Thread(target=program, args=(i,)) for i in (1, 2, 3)]
    for t in th:
        t.start()
    for t in th:
        t.join(30)
    assert not errors, errors
    for i in (1, 2, 3):
        assert np.array_equal(results[i], np.full(200, 3.0 * i, np.float32))
    tr = s.trace()
    dec = assert_trace_matches_replay(s.desc, tr)
    assert (dec["kind"] == oracle.D_ADMIT).sum() == 3 and s.stats().free_bytes == 1000


def test_threads_of_one_runtime_do_not_block_each_other_while_one_waits():
    # one runtime, two threads: the second launch does not fit until the first task's object is
    # freed, and the free has to get through the runtime while the launch is waiting in it
    s = mgb.Sched(backend=mgb.MGB_BACKEND_NULL, mem_cap_bytes=1000, granule_cus=8)
    z = mgb.Lazy(s)
    rc, a = z.malloc(800)
    rc, b = z.malloc(800)
    rc, real, pl = z.launch_prepare(1, [a], (1, 1, 1), (64, 1, 1))
    assert rc == 0
    out = {}

    def second():
        out["rc"], out["real"], out["pl"] = z.launch_prepare(2, [b], (1, 1, 1), (64, 1, 1), timeout_ns=20_000_000_000)

    th = threading.Thread(target=second)
    th.start()
    for _ in range(2000):                       # until the second probe is queued
        if s.stats().n_waiting == 1:
            break
        threading.Event().wait(0.001)
    assert s.stats().n_waiting == 1
    assert z.free(a) == 0                       # would wait forever if the waiter held the runtime's lock
    th.join(30)
    assert not th.is_alive() and out["rc"] == 0 and out["real"][0] != 0
    assert z.free(b) == 0 and z.destroy() == 0
    assert_trace_matches_replay(s.desc, s.trace())
    assert s.destroy() == 0


def test_copy_back_of_a_window_of_an_unbound_object():
    # reads of a never-bound object see the recorded writes clipped to the window asked for
    s = mgb.Sched(backend=mgb.MGB_BACKEND_NULL, granule_cus=8)
    z = mgb.Lazy(s)
    rc, a = z.malloc(1 << 30)                   # large: the read must not materialise the object
    src = np.arange(64, dtype=np.uint8)
    assert z.memset(a, 7, 1 << 30) == 0
    assert z.memcpy_h2d(a + 100, src.ctypes.data, 64) == 0
    assert z.memset(a + 120, 9, 8) == 0
    got = np.zeros(80, np.uint8)
    assert z.memcpy_d2h(got.ctypes.data, a + 90, 80) == 0
    want = np.full(80, 7, np.uint8)
    want[10:74] = src
    want[30:38] = 9
    assert np.array_equal(got, want)
    assert z.free(a) == 0 and z.destroy() == 0 and s.destroy() == 0


def test_allocation_failure_after_admission_rolls_the_ledger_back():
    # the task is admitted (the cap allows it), then binding its second object fails in the
    # allocator: what was bound is released, the ticket completed, the ledger whole again
    cap = 1 << 41
    s = mgb.Sched(backend=mgb.MGB_BACKEND_NULL, granule_cus=8, mem_cap_bytes=cap)
    z = mgb.Lazy(s)
    rc, small = z.malloc(1000)
    rc, huge = z.malloc((1 << 40) - 1)                   # no host gives this to the null backend
    src = np.arange(250, dtype=np.float32)
    assert z.memcpy_h2d(small, src.ctypes.data, 1000) == 0
    rc, real, pl = z.launch_prepare(1, [small, huge], (1, 1, 1), (64, 1, 1))
    if rc == 0:
        pytest.skip("the host handed out a terabyte of address space")
    assert rc == mgb.MGB_E_BACKEND
    st, zs = s.stats(), z.stats()
    assert (st.free_bytes, st.n_running, st.n_waiting) == (cap, 0, 0)
    assert (zs.n_bound, zs.n_tasks, zs.n_objects) == (0, 0, 2)
    # the objects are still there, unbound, with their recorded writes: a smaller launch works
    rc, real, pl = z.launch_prepare(2, [small], (1, 1, 1), (64, 1, 1))
    assert rc == 0 and np.array_equal(_f32(_real_view(real[0], 1000), 250), src)
    assert z.free(small) == 0 and z.free(huge) == 0 and z.destroy() == 0
    assert_trace_matches_replay(s.desc, s.trace())
    assert s.destroy() == 0


def test_a_launch_that_times_out_while_it_is_being_admitted_leaks_nothing():
    # A launch waits for memory with a short timeout while another thread frees that memory at about
    # the same moment.  Whichever way each round goes (timed out and withdrawn, admitted, or admitted
    # in the gap between the two), the scheduler must end up empty.
    import random
    import time
    s = mgb.Sched(backend=mgb.MGB_BACKEND_NULL, mem_cap_bytes=100)
    z = mgb.Lazy(s)
    rnd = random.Random(3)
    got = {mgb.MGB_OK: 0, mgb.MGB_TIMEOUT: 0}
    for it in range(300):
        rc, x = z.malloc(60)
        rc, real, pl = z.launch_prepare(2 * it, [x], (1, 1, 1), (64, 1, 1))
        assert rc == mgb.MGB_OK
        rc, y = z.malloc(60)
        out = []
        th = threading.Thread(target=lambda: out.append(z.launch_prepare(2 * it + 1, [y], (1, 1, 1), (64, 1, 1),
                                                                         timeout_ns=rnd.choice([0, 20_000, 60_000, 200_000]))[0]))
        th.start()
        time.sleep(rnd.choice([0, 2e-5, 6e-5, 1e-4]))
        assert z.free(x) == mgb.MGB_OK
        th.join(10)
        assert out and out[0] in (mgb.MGB_OK, mgb.MGB_TIMEOUT), out
        got[out[0]] += 1
        assert z.free(y) == mgb.MGB_OK
        st = s.stats()
        assert (st.n_running, st.n_waiting, st.free_bytes) == (0, 0, 100), (it, out)
    assert got[mgb.MGB_OK] > 0
    assert_trace_matches_replay(s.desc, s.trace())
    assert z.destroy() == mgb.MGB_OK and s.destroy() == mgb.MGB_OK
