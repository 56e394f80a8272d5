"""Client programs that the multi-process tests start as separate processes (not collected by pytest)."""
import sys
import time


def _client(name):
    import paper_2107_08538_amd as mgb
    return mgb, mgb.Client(name)


def storm(name, seed, n_tasks):
    """Runs n_tasks small tasks one after the other; exits 0 if every call behaved."""
    import numpy as np
    mgb, c = _client(name)
    rng = np.random.default_rng(seed)
    for i in range(n_tasks):
        mem = int(rng.integers(100, 600))
        rc, pl = c.probe(seed * 1000 + i, mem, (int(rng.integers(1, 2000)), 1, 1), (256, 1, 1))
        if rc == mgb.MGB_WAIT:
            rc, pl = c.wait(pl.ticket)
        assert rc == mgb.MGB_OK, rc
        assert pl.stream is None and pl.granule_mask != 0 and any(pl.cu_mask)
        time.sleep(float(rng.uniform(0, 0.004)))
        if rng.random() < 0.3:
            assert c.grow(pl.ticket, int(rng.integers(1, 200))) in (mgb.MGB_OK, mgb.MGB_E_BUSY)
        assert c.complete(pl.ticket) == mgb.MGB_OK
    assert c.disconnect() == mgb.MGB_OK


def hold_and_die(name, mem):
    """Takes memory and dies without giving it back."""
    import os
    mgb, c = _client(name)
    rc, pl = c.probe(666, mem, (8, 1, 1), (64, 1, 1))
    assert rc == mgb.MGB_OK
    rc, pl2 = c.probe(667, mem, (8, 1, 1), (64, 1, 1))        # does not fit beside the first: queued
    assert rc == mgb.MGB_WAIT
    print("holding", flush=True)
    time.sleep(0.3)
    os._exit(0)


def gpu_task(name, kind, seed):
    """One real task on this process's own masked stream; checks its result against the checker."""
    import ctypes as C
    import numpy as np
    import torch
    import oracle
    import workloads as W
    mgb, c = _client(name)
    P = lambda t: C.c_void_p(t.data_ptr())
    if kind == "jacobi":
        n, it = 512, 20
        u = W.jacobi_field(seed, n)
        u0 = torch.from_numpy(u).cuda()
        u1 = u0.clone()
        mem, grid, block = mgb.probe_of(mgb.mgb_jacobi_probe, n, it)
        run = lambda st: mgb.mgb_jacobi_enqueue(st, P(u0), P(u1), n, it)
    else:
        n = 384
        a, b = W.gemm_operands_f32(seed, n, n, n)
        A, B, Cc = torch.from_numpy(a).cuda(), torch.from_numpy(b).cuda(), torch.zeros(n, n, device="cuda")
        mem, grid, block = mgb.probe_of(mgb.mgb_gemm_f32_probe, n, n, n)
        run = lambda st: mgb.mgb_gemm_f32_enqueue(st, P(A), P(B), P(Cc), n, n, n)
    torch.cuda.synchronize()
    rc, pl = c.probe(seed, mem, grid, block)
    if rc == mgb.MGB_WAIT:
        rc, pl = c.wait(pl.ticket)
    assert rc == mgb.MGB_OK, rc
    rc, st = c.stream(pl)
    assert rc == mgb.MGB_OK and st.value
    # where do workgroups on this stream run?  only on the CUs of the granted mask
    out = torch.zeros(2048, dtype=torch.int32, device="cuda")
    assert mgb.mgb_cu_trace_enqueue(st, P(out), 2048) == 0
    assert run(st) == 0
    torch.cuda.synchronize()
    cus = set(out.cpu().numpy().tolist())
    want = sum(bin(w).count("1") for w in pl.cu_mask)
    assert len(cus) <= want and len(cus) >= min(want, 8), (len(cus), want)
    if kind == "jacobi":
        assert np.array_equal(u0.cpu().numpy(), oracle.jacobi_f32(u, it))
    else:
        got = Cc.cpu().numpy().astype(np.float64)
        assert (np.abs(got - oracle.gemm_f32(a, b)) / oracle.gemm_abs_f32(a, b)).max() <= 1e-4
    assert c.complete(pl.ticket) == mgb.MGB_OK
    assert c.disconnect() == mgb.MGB_OK
    print("ok", kind, len(cus), want, flush=True)


if __name__ == "__main__":
    import os
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    fn = sys.argv[1]
    if fn == "storm":
        storm(sys.argv[2], int(sys.argv[3]), int(sys.argv[4]))
    elif fn == "hold_and_die":
        hold_and_die(sys.argv[2], int(sys.argv[3]))
    elif fn == "gpu_task":
        gpu_task(sys.argv[2], sys.argv[3], int(sys.argv[4]))
    else:
        sys.exit(9)
