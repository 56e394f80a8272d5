"""The kernels at the largest shapes their entry points accept (65536 rows / columns): outputs of
16 GiB, whose byte offsets need more than 32 bits.  Checked on sampled entries, whole border rows
and columns included, that the serial checker computes one by one."""
import ctypes as C

import numpy as np
import pytest

import oracle
import workloads as W

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

import paper_2107_08538_amd as mgb  # noqa: E402

DEV = "cuda:0"
N = 65536


def P(t):
    return C.c_void_p(t.data_ptr())


def _need(gib):
    free_b, _ = torch.cuda.mem_get_info()
    if free_b < (gib + 4) << 30:
        pytest.skip("needs %d GiB of free device memory" % gib)


def _sample(rng):
    rows = rng.integers(0, N, 8192).astype(np.uint32)
    cols = rng.integers(0, N, 8192).astype(np.uint32)
    every = np.arange(N, dtype=np.uint32)
    last = np.full(N, N - 1, dtype=np.uint32)
    # random entries, the first and the last row, the last column
    return (np.concatenate([rows, np.zeros(N, np.uint32), last, every]),
            np.concatenate([cols, every, every, last]))


def test_gemm_f32_65536_x_65536():
    _need(17)
    k = 16
    a, b = W.gemm_operands_f32(11, N, N, k)
    A, B = torch.from_numpy(a).to(DEV), torch.from_numpy(b).to(DEV)
    Cd = torch.full((N, N), float("nan"), device=DEV)
    assert mgb.mgb_gemm_f32_enqueue(None, P(A), P(B), P(Cd), N, N, k) == 0, mgb.mgb_last_error()
    torch.cuda.synchronize()
    rows, cols = _sample(np.random.default_rng(1))
    got = Cd[torch.from_numpy(rows.astype(np.int64)).to(DEV), torch.from_numpy(cols.astype(np.int64)).to(DEV)]
    got = got.cpu().numpy().astype(np.float64)
    ref, den = oracle.gemm_f32_entries(a, b, rows, cols)
    assert (np.abs(got - ref) / den).max() <= 1e-4
    assert not bool(torch.isnan(Cd[::4099]).any())           # every 4099th row: nothing left unwritten


def test_gemm_bf16_65536_x_65536():
    _need(17)
    k = 32
    ab, bb = W.gemm_operands_bf16(12, N, N, k)
    A = torch.from_numpy(ab.view("int16")).to(DEV)
    B = torch.from_numpy(bb.view("int16")).to(DEV)
    Cd = torch.full((N, N), float("nan"), device=DEV)
    assert mgb.mgb_gemm_bf16_enqueue(None, P(A), P(B), P(Cd), N, N, k) == 0, mgb.mgb_last_error()
    torch.cuda.synchronize()
    rows, cols = _sample(np.random.default_rng(2))
    got = Cd[torch.from_numpy(rows.astype(np.int64)).to(DEV), torch.from_numpy(cols.astype(np.int64)).to(DEV)]
    got = got.cpu().numpy().astype(np.float64)
    ref = oracle.gemm_bf16_entries(ab, bb, rows, cols)
    assert np.linalg.norm(got - ref) / np.linalg.norm(ref) <= 1e-2
    assert not bool(torch.isnan(Cd[::4099]).any())


def test_jacobi_65536_squared():
    _need(33)
    it = 3
    gen = torch.Generator(device=DEV)
    gen.manual_seed(13)
    u0 = torch.rand(N, N, device=DEV, generator=gen)
    u0[0, :] = 0
    u0[-1, :] = 0
    u0[:, 0] = 0
    u0[:, -1] = 0
    u1 = u0.clone()
    # a cell after `it` sweeps depends on the initial cells within distance `it`: keep those patches
    rng = np.random.default_rng(3)
    pts = [(1, 1), (N - 2, N - 2), (1, N - 2), (N - 2, 1), (N // 2, N // 2), (N - 2, 40000), (32768, 1)]
    pts += [(int(r), int(c)) for r, c in zip(rng.integers(1, N - 1, 40), rng.integers(1, N - 1, 40))]
    side = 2 * it + 3
    patches = []
    for (r, c) in pts:
        r0 = min(max(0, r - it - 1), N - side)
        c0 = min(max(0, c - it - 1), N - side)
        patches.append((r, c, r0, c0, u0[r0:r0 + side, c0:c0 + side].cpu().numpy().copy()))
    assert mgb.mgb_jacobi_enqueue(None, P(u0), P(u1), N, it) == 0, mgb.mgb_last_error()
    torch.cuda.synchronize()
    res = u0 if it % 2 == 0 else u1
    for (r, c, r0, c0, patch) in patches:
        # the checker holds the window's rim fixed: true where it is the grid's own ring, and elsewhere
        # the rim is at least it + 1 cells from (r, c), out of reach in `it` sweeps
        want = oracle.jacobi_f32(np.ascontiguousarray(patch), it)[r - r0, c - c0]
        assert float(res[r, c]) == float(want), (r, c)
    assert float(res[0].abs().max()) == 0.0 and float(res[:, -1].abs().max()) == 0.0    # the ring stays
