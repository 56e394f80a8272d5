"""mgb_bfs_enqueue_static (the traversal with its work area in the library's static device array,
for callers that cannot allocate) against mgb_bfs_enqueue with a caller buffer: levels and depth
bit for bit, on two calls in a row that share the array, the second on a smaller graph, and
against the CPU checker.  Collected last: a failure here must not hide another test."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle
import paper_2107_08538_amd as mgb
import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def P(t):
    return C.c_void_p(t.data_ptr())


def _both(rp, ci, source):
    n = rp.size - 1
    RP, CI = torch.from_numpy(rp).to(DEV), torch.from_numpy(ci).to(DEV)
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    out = []
    for static in (False, True):
        lev = torch.full((n,), -7, dtype=torch.int32, device=DEV)
        depth = C.c_uint32(0)
        if static:
            rc = mgb.mgb_bfs_enqueue_static(st, P(RP), P(CI), n, source, P(lev), C.byref(depth))
        else:
            work = torch.zeros(mgb.mgb_bfs_work_bytes(n), dtype=torch.uint8, device=DEV)
            rc = mgb.mgb_bfs_enqueue(st, P(RP), P(CI), n, source, P(lev), P(work), C.byref(depth))
        assert rc == 0, mgb.mgb_last_error()
        torch.cuda.synchronize()
        out.append((lev.cpu().numpy(), depth.value))
    return out


def test_static_work_area_matches_caller_buffer_on_two_calls_in_a_row():
    # second call smaller: queues, bitmaps and counters of the first are still in the array
    for seed, n, deg, source in ((11, (1 << 20) + 4097, 12, 5), (12, 70001, 6, 69000)):
        print("bfs static: seed %d n %d degree %s" % (seed, n, deg), flush=True)
        rp, ci = W.er_graph_csr(seed, n, deg)
        (want, d0), (got, d1) = _both(rp, ci, source)
        assert np.array_equal(got, want)
        assert d0 == d1
        assert np.array_equal(got, oracle.bfs(rp, ci, source))


def test_static_work_area_rejects_what_does_not_fit():
    t = torch.zeros(16, dtype=torch.int32, device=DEV)
    rc = mgb.mgb_bfs_enqueue_static(None, P(t), P(t), (1 << 22) + 1, 0, P(t), None)
    assert rc == mgb.MGB_E_TOO_BIG
    assert b"2^22" in mgb.mgb_last_error()
    assert mgb.mgb_bfs_enqueue_static(None, P(t), P(t), 4, 4, P(t), None) == mgb.MGB_E_INVAL     # source >= n
