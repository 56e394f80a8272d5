"""Lazy runtime on the GPU: tasks whose footprint is discovered at the launch (Sec. III-A) give the
same results as the checker and the same footprints as the declared probes."""
import ctypes as C
import threading

import numpy as np
import pytest

import oracle
import workloads as W
from helpers import assert_trace_matches_replay

pytestmark = pytest.mark.gpu

import paper_2107_08538_amd as mgb  # noqa: E402


def _h2d(z, pseudo, arr):
    arr = np.ascontiguousarray(arr)
    assert z.memcpy_h2d(pseudo, arr.ctypes.data, arr.nbytes) == 0


def _d2h(z, pseudo, shape, dtype):
    out = np.empty(shape, dtype=dtype)
    assert z.memcpy_d2h(out.ctypes.data, pseudo, out.nbytes) == 0
    return out


def test_gemm_task_built_lazily_matches_checker_and_declared_footprint():
    m, n, k = 300, 264, 200
    a, b = W.gemm_operands_f32(3, m, n, k)
    s = mgb.Sched()
    z = mgb.Lazy(s)
    pa, pb, pc = (z.malloc(x)[1] for x in (a.nbytes, b.nbytes, m * n * 4))
    _h2d(z, pa, a)
    _h2d(z, pb, b)
    a[:] = 0                                           # the copy kept its own bytes
    assert len(s.trace()) == 0
    mem, grid, block = mgb.probe_of(mgb.mgb_gemm_f32_probe, m, n, k)
    rc, real, pl = z.launch_prepare(11, [pa, pb, pc], grid, block, wg_per_cu=mgb.mgb_gemm_f32_residency(m, n, k))
    assert rc == 0 and pl.stream and all(real)
    assert mgb.mgb_gemm_f32_enqueue(pl.stream, real[0], real[1], real[2], m, n, k) == 0
    got = _d2h(z, pc, (m, n), np.float32).astype(np.float64)
    a, b = W.gemm_operands_f32(3, m, n, k)
    ref, den = oracle.gemm_f32(a, b), oracle.gemm_abs_f32(a, b)
    assert (np.abs(got - ref) / den).max() <= 1e-4
    tr = s.trace()
    probes = tr[tr["kind"] == mgb.MGB_EV_PROBE]
    assert len(probes) == 1 and int(probes[0]["mem_bytes"]) == mem          # discovered = declared
    for p in (pa, pb, pc):
        assert z.free(p) == 0
    assert s.stats().n_running == 0 and z.destroy() == 0
    assert_trace_matches_replay(s.desc, s.trace())
    assert s.destroy() == 0


def test_kernels_sharing_buffers_form_one_task_that_grows():
    # Jacobi sweeps on (u0, u1), then C = U * U with a new C: the second launch joins the task
    n, it = 256, 6
    u = W.jacobi_field(5, n)
    s = mgb.Sched()
    z = mgb.Lazy(s)
    p0, p1 = z.malloc(u.nbytes)[1], z.malloc(u.nbytes)[1]
    _h2d(z, p0, u)
    _h2d(z, p1, u)
    mem_j, grid_j, block_j = mgb.probe_of(mgb.mgb_jacobi_probe, n, it)
    rc, real, pl = z.launch_prepare(1, [p0, p1], grid_j, block_j)
    assert rc == 0
    assert mgb.mgb_jacobi_enqueue(pl.stream, real[0], real[1], n, it) == 0
    pc = z.malloc(n * n * 4)[1]
    mem_g, grid_g, block_g = mgb.probe_of(mgb.mgb_gemm_f32_probe, n, n, n)
    rc, real2, pl2 = z.launch_prepare(1, [p0, p0, pc], grid_g, block_g)
    assert rc == 0 and pl2.stream == pl.stream and real2[0] == real[0] and pl2.ticket == pl.ticket
    assert mgb.mgb_gemm_f32_enqueue(pl2.stream, real2[0], real2[1], real2[2], n, n, n) == 0
    ref_u = oracle.jacobi_f32(u, it)                   # it is even: the result is in u0
    assert np.array_equal(_d2h(z, p0, (n, n), np.float32), ref_u)
    got = _d2h(z, pc, (n, n), np.float32).astype(np.float64)
    ref, den = oracle.gemm_f32(ref_u, ref_u), oracle.gemm_abs_f32(ref_u, ref_u)
    assert (np.abs(got - ref) / np.maximum(den, 1e-30)).max() <= 1e-4
    tr = s.trace()
    assert int(tr[tr["kind"] == mgb.MGB_EV_PROBE][0]["mem_bytes"]) == mem_j
    grows = tr[tr["kind"] == mgb.MGB_EV_GROW]
    assert len(grows) == 1 and int(grows[0]["mem_bytes"]) == n * n * 4
    assert s.stats().free_bytes == s.desc.mem_cap_bytes - mem_j - n * n * 4
    for p in (p0, p1, pc):
        assert z.free(p) == 0
    assert s.stats().free_bytes == s.desc.mem_cap_bytes and z.destroy() == 0
    assert_trace_matches_replay(s.desc, s.trace())
    assert s.destroy() == 0


def test_lazy_clients_queue_for_memory_and_all_finish():
    # four programs, each its own lazy instance; the cap holds two of their tasks at a time
    n = 512
    one = 3 * n * n * 4
    s = mgb.Sched(mem_cap_bytes=2 * one + 1000)
    results, errors = {}, []

    def program(i):
        try:
            a, b = W.gemm_operands_f32(20 + i, n, n, n)
            z = mgb.Lazy(s)
            pa, pb, pc = (z.malloc(n * n * 4)[1] for _ in range(3))
            _h2d(z, pa, a)
            _h2d(z, pb, b)
            mem, grid, block = mgb.probe_of(mgb.mgb_gemm_f32_probe, n, n, n)
            rc, real, pl = z.launch_prepare(i, [pa, pb, pc], grid, block)
            assert rc == 0, rc
            assert mgb.mgb_gemm_f32_enqueue(pl.stream, real[0], real[1], real[2], n, n, n) == 0
            results[i] = (_d2h(z, pc, (n, n), np.float32), a, b)
            for p in (pa, pb, pc):
                assert z.free(p) == 0
            assert z.destroy() == 0
        except Exception as e:   # noqa: BLE001
            errors.append((i, repr(e)))

    th = [threading.Thread(target=program, args=(i,)) for i in range(4)]
    for t in th:
        t.start()
    for t in th:
        t.join(120)
    assert not errors, errors
    for i, (got, a, b) in results.items():
        ref, den = oracle.gemm_f32(a, b), oracle.gemm_abs_f32(a, b)
        assert (np.abs(got.astype(np.float64) - ref) / den).max() <= 1e-4, i
    tr = s.trace()
    dec = assert_trace_matches_replay(s.desc, tr)
    assert (dec["kind"] == oracle.D_ADMIT).sum() == 4 and (dec["kind"] == oracle.D_WAIT).sum() >= 1
    assert s.stats().free_bytes == s.desc.mem_cap_bytes
    assert s.destroy() == 0
