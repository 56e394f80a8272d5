"""Parity of every HIP task kernel with the CPU checker, through the C ABI.

Tolerances (written where used): Jacobi max relative error <= 1e-5 (and bit-exact against the
fixed-association fp32 definition); fp32 GEMM max componentwise error <= 1e-4; bf16 GEMM / conv
relative Frobenius error <= 1e-2; BFS levels bit-exact."""
import ctypes as C

import numpy as np
import pytest

import oracle
import workloads as W
from helpers import frobenius_rel

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

import paper_2107_08538_amd as mgb  # noqa: E402

DEV = "cuda:0"
u32 = C.c_uint32


def P(t):
    return C.c_void_p(t.data_ptr())


def sync():
    torch.cuda.synchronize()


# ------------------------------------------------------------------ Jacobi
def run_jacobi(u, iters):
    n = u.shape[0]
    u0 = torch.from_numpy(u).to(DEV)
    u1 = u0.clone()
    rc = mgb.mgb_jacobi_enqueue(None, P(u0), P(u1), n, iters)
    assert rc == 0, mgb.mgb_last_error()
    sync()
    return (u0 if iters % 2 == 0 else u1).cpu().numpy()


@pytest.mark.parametrize("n,iters", [(3, 1), (4, 3), (5, 2), (64, 5), (77, 6), (100, 3), (512, 20),
                                     (1028, 4), (1100, 5), (2050, 3), (130, 0), (2048, 7)])
def test_jacobi_bit_exact_and_within_tolerance(n, iters):
    u = W.jacobi_field(n + iters, n)
    got = run_jacobi(u, iters)
    assert np.array_equal(got, oracle.jacobi_f32(u, iters))          # same association => same bits
    ref = oracle.jacobi_f64(u, iters)
    assert np.all(got[0, :] == 0) and np.all(got[-1, :] == 0)        # ring exactly zero
    assert np.all(got[:, 0] == 0) and np.all(got[:, -1] == 0)
    if n > 2 and iters > 0:
        inner = ref[1:-1, 1:-1]
        err = np.abs(got.astype(np.float64) - ref)[1:-1, 1:-1]
        pos = inner > 0
        assert np.all(err[~pos] == 0)                                # exact zeros stay exact
        if pos.any():
            assert (err[pos] / inner[pos]).max() <= 1e-5


def test_jacobi_nonzero_ring_and_constant_field():
    n = 260
    u = np.full((n, n), 0.3, dtype=np.float32)
    assert np.array_equal(run_jacobi(u, 9), u)                       # constant field is a fixed point
    rng = np.random.default_rng(0)
    u = rng.random((n, n), dtype=np.float32)                         # random ring stays and feeds in
    assert np.array_equal(run_jacobi(u, 4), oracle.jacobi_f32(u, 4))


def test_jacobi_streaming_keeps_a_nonzero_ring():
    # the streaming launches (2048 columns and more, five to eight sweeps) with values on the ring
    n = 4100
    rng = np.random.default_rng(1)
    u = rng.random((n, n), dtype=np.float32)
    got = run_jacobi(u, 7)
    want = oracle.jacobi_f32(u, 7)
    assert np.array_equal(got, want)
    assert np.array_equal(got[0], u[0]) and np.array_equal(got[:, -1], u[:, -1])


def test_jacobi_full_size_mix16_task():
    n, iters = 4096, 100
    u = W.jacobi_field(123, n)
    got = run_jacobi(u, iters)
    assert np.array_equal(got, oracle.jacobi_f32(u, iters))


@pytest.mark.parametrize("n,iters,launches", [(8200, 5, 1), (8192, 12, 2), (8444, 17, 3), (4100, 7, 1), (4096, 13, 3),
                                              (5000, 21, 3), (4344, 32, 4), (4096, 6, 2),
                                              (2048, 8, 2), (2052, 7, 1), (2816, 15, 3), (3000, 50, 8), (3964, 24, 4)])
def test_jacobi_streaming_launches_of_five_to_eight_sweeps(n, iters, launches):
    # from 2048 columns on a launch fuses up to eight sweeps; launches of five and more stream down
    # strips of 240 columns in runs of 40 rows (ragged last strips and runs in every case here),
    # launches of up to four (13 = 5 + 4 + 4, 6 = 3 + 3) use the window kernel
    u = W.jacobi_field(321, n)
    assert mgb.mgb_jacobi_launch_count(n, iters) == launches
    got = run_jacobi(u, iters)
    assert np.array_equal(got, oracle.jacobi_f32(u, iters))


def test_jacobi_large_eigenmode_property():
    # 16384^2 (the largest task size): an eigenmode of the sweep must come back scaled by lambda^k
    n, k, p, q = 16384, 10, 3, 5
    i = np.arange(n, dtype=np.float64)
    s1, s2 = np.sin(np.pi * p * i / (n - 1)), np.sin(np.pi * q * i / (n - 1))
    u = np.outer(s1, s2).astype(np.float32)
    u[0, :] = u[-1, :] = 0
    u[:, 0] = u[:, -1] = 0
    got = run_jacobi(u, k)
    lam = 0.5 * (np.cos(np.pi * p / (n - 1)) + np.cos(np.pi * q / (n - 1)))
    rows = np.array([1, 2, 1000, 8191, 8192, 16000, 16382])
    want = lam ** k * np.outer(s1[rows], s2)
    assert np.abs(got[rows] - want).max() <= 2e-6
    assert np.all(got[0] == 0) and np.all(got[:, -1] == 0)


def test_jacobi_rejects_bad_arguments():
    t = torch.zeros(16, device=DEV)
    assert mgb.mgb_jacobi_enqueue(None, P(t), P(t), 4, 1) == mgb.MGB_E_INVAL          # same buffer
    assert mgb.mgb_jacobi_enqueue(None, None, P(t), 4, 1) == mgb.MGB_E_INVAL
    assert mgb.mgb_jacobi_enqueue(None, P(t), P(t[1:]), 3, 1) == mgb.MGB_E_INVAL      # misaligned
    t2 = torch.zeros(16, device=DEV)
    assert mgb.mgb_jacobi_enqueue(None, P(t), P(t2), 2, 1) == mgb.MGB_E_UNSUPPORTED


# ------------------------------------------------------------------ GEMM fp32
def run_gemm_f32(a, b):
    m, k = a.shape
    n = b.shape[1]
    A, B = torch.from_numpy(a).to(DEV), torch.from_numpy(b).to(DEV)
    Cd = torch.full((m, n), float("nan"), device=DEV)
    assert mgb.mgb_gemm_f32_enqueue(None, P(A), P(B), P(Cd), m, n, k) == 0, mgb.mgb_last_error()
    sync()
    return Cd.cpu().numpy()


@pytest.mark.parametrize("m,n,k", [(1, 1, 1), (128, 128, 16), (100, 70, 33), (129, 257, 17),
                                   (256, 256, 256), (384, 128, 48), (512, 384, 1000), (130, 128, 16),
                                   (128, 128, 15), (31, 513, 64),
                                   # k % 16 == 0 and n % 4 == 0: the DMA-ring kernel.  64 x 64 tiles with ragged
                                   # rows / columns and fewer k tiles than ring stages ...
                                   (1, 4, 16), (64, 64, 16), (200, 132, 48), (1000, 1004, 160),
                                   # ... and 128 x 128 tiles (at least 128 of them), ragged and full
                                   (1408, 1540, 64), (1500, 1412, 112), (2048, 1024, 256),
                                   # ... and 256 x 256 tiles (exactly one round of 256 of them, ragged); with a
                                   # few tiles more than a round the 128 x 128 kernel is taken (the last two)
                                   (3900, 4092, 32), (4000, 4096, 48), (4096, 4100, 32), (4000, 4352, 48)])
def test_gemm_f32_componentwise_error(m, n, k):
    a, b = W.gemm_operands_f32(m * 7 + k, m, n, k)
    got = run_gemm_f32(a, b)
    ref, den = oracle.gemm_f32(a, b), oracle.gemm_abs_f32(a, b)
    assert (np.abs(got.astype(np.float64) - ref) / den).max() <= 1e-4
    assert np.abs(got - ref).max() / np.abs(ref).max() <= 1e-5


def test_gemm_f32_unaligned_operands_take_the_staged_kernel():
    m, n, k = 200, 132, 48
    a, b = W.gemm_operands_f32(12, m, n, k)
    A = torch.zeros(m * k + 4, device=DEV)
    A[1:1 + m * k] = torch.from_numpy(a.ravel()).to(DEV)                  # 4-byte aligned only
    B = torch.from_numpy(b).to(DEV)
    Cd = torch.full((m, n), float("nan"), device=DEV)
    assert mgb.mgb_gemm_f32_enqueue(None, C.c_void_p(A.data_ptr() + 4), P(B), P(Cd), m, n, k) == 0
    sync()
    ref, den = oracle.gemm_f32(a, b), oracle.gemm_abs_f32(a, b)
    assert (np.abs(Cd.cpu().numpy().astype(np.float64) - ref) / den).max() <= 1e-4


def test_gemm_f32_identity_and_permutation_exact():
    a, _ = W.gemm_operands_f32(3, 256, 256, 256)
    eye = np.eye(256, dtype=np.float32)
    assert np.array_equal(run_gemm_f32(a, eye), a)
    perm = np.random.default_rng(1).permutation(256)
    assert np.array_equal(run_gemm_f32(eye[perm], a), a[perm])


def test_gemm_f32_full_size_sampled_and_freivalds():
    n = 4096
    a, b = W.gemm_operands_f32(77, n, n, n)
    got = run_gemm_f32(a, b).astype(np.float64)
    rng = np.random.default_rng(5)
    rows = rng.integers(0, n, 4096).astype(np.uint32)
    cols = rng.integers(0, n, 4096).astype(np.uint32)
    rows[:4], cols[:4] = [0, 0, n - 1, n - 1], [0, n - 1, 0, n - 1]
    ref, den = oracle.gemm_f32_entries(a, b, rows, cols)
    assert (np.abs(got[rows, cols] - ref) / den).max() <= 1e-4
    # Freivalds: C x = A (B x) for random x, all 16.7M entries covered at O(n^2) cost
    x = rng.standard_normal(n)
    lhs = got @ x
    a64, b64 = a.astype(np.float64), b.astype(np.float64)
    rhs = a64 @ (b64 @ x)
    bound = np.abs(a64) @ (np.abs(b64) @ np.abs(x))
    assert (np.abs(lhs - rhs) / bound).max() <= 1e-4


# ------------------------------------------------------------------ GEMM bf16
def run_gemm_bf16(ab, bb):
    m, k = ab.shape
    n = bb.shape[1]
    A = torch.from_numpy(ab.view(np.int16)).to(DEV)
    B = torch.from_numpy(bb.view(np.int16)).to(DEV)
    Cd = torch.full((m, n), float("nan"), device=DEV)
    assert mgb.mgb_gemm_bf16_enqueue(None, P(A), P(B), P(Cd), m, n, k) == 0, mgb.mgb_last_error()
    sync()
    return Cd.cpu().numpy()


@pytest.mark.parametrize("m,n,k", [(1, 1, 1), (128, 128, 32), (128, 128, 64), (100, 70, 33),
                                   (129, 257, 17), (256, 256, 256), (384, 128, 96), (512, 384, 1000),
                                   # k % 32 == 0 and n % 8 == 0: the 256 x 256 DMA-ring kernel, with
                                   # ragged rows / columns, fewer k tiles than ring stages, several tiles
                                   (1, 8, 32), (256, 8, 64), (300, 520, 64), (513, 264, 2048),
                                   (1024, 1024, 32), (768, 512, 96), (2000, 1096, 1056),
                                   # at least 128 tiles of 256 x 256: the big-tile variant (the others above take 128 x 128)
                                   (2816, 2824, 64), (3000, 2816, 96),
                                   # k % 64 == 0: A travels 64 deep through a ring of three stages; fewer pieces
                                   # than stages, as many, more, ragged rows / columns, both tile sizes
                                   (256, 264, 128), (260, 256, 192), (520, 392, 704), (1000, 1032, 1088),
                                   (2830, 2816, 448), (2816, 2832, 128)])
def test_gemm_bf16_frobenius_error(m, n, k):
    ab, bb = W.gemm_operands_bf16(m + 3 * k, m, n, k)
    got = run_gemm_bf16(ab, bb)
    ref = oracle.gemm_bf16(ab, bb)
    assert frobenius_rel(got, ref) <= 1e-2
    assert frobenius_rel(got, ref) <= 1e-5          # fp32 accumulation of exact products


def test_gemm_bf16_unaligned_operands_take_the_staged_kernel():
    m, n, k = 200, 264, 96
    ab, bb = W.gemm_operands_bf16(11, m, n, k)
    A = torch.zeros(m * k + 8, dtype=torch.int16, device=DEV)
    A[1:1 + m * k] = torch.from_numpy(ab.view(np.int16).ravel()).to(DEV)      # 2-byte aligned only
    B = torch.from_numpy(bb.view(np.int16)).to(DEV)
    Cd = torch.full((m, n), float("nan"), device=DEV)
    assert mgb.mgb_gemm_bf16_enqueue(None, C.c_void_p(A.data_ptr() + 2), P(B), P(Cd), m, n, k) == 0
    sync()
    assert frobenius_rel(Cd.cpu().numpy(), oracle.gemm_bf16(ab, bb)) <= 1e-5


@pytest.mark.parametrize("k", [160, 448])           # depth-32 ring for both operands; A 64 deep
def test_gemm_bf16_layout_exact_small_integers(k):
    # small integers are exact in bf16 and their dot products exact in fp32: any operand
    # layout mistake shows as a wrong integer
    rng = np.random.default_rng(2)
    a = rng.integers(-4, 5, (256, k)).astype(np.float32)
    b = rng.integers(-4, 5, (k, 384)).astype(np.float32)
    got = run_gemm_bf16(W.f32_to_bf16_bits(a), W.f32_to_bf16_bits(b))
    assert np.array_equal(got, a @ b)


def test_gemm_bf16_full_size_sampled():
    n = 4096
    ab, bb = W.gemm_operands_bf16(99, n, n, n)
    got = run_gemm_bf16(ab, bb).astype(np.float64)
    rng = np.random.default_rng(6)
    rows = rng.integers(0, n, 2048).astype(np.uint32)
    cols = rng.integers(0, n, 2048).astype(np.uint32)
    ref = oracle.gemm_bf16_entries(ab, bb, rows, cols)
    assert np.linalg.norm(got[rows, cols] - ref) / np.linalg.norm(ref) <= 1e-2
    x = rng.standard_normal(n)
    a64 = W.bf16_bits_to_f32(ab).astype(np.float64)
    b64 = W.bf16_bits_to_f32(bb).astype(np.float64)
    lhs, rhs = got @ x, a64 @ (b64 @ x)
    assert np.linalg.norm(lhs - rhs) / np.linalg.norm(rhs) <= 1e-2


# ------------------------------------------------------------------ conv
def run_conv(x, w, stride, out_f32):
    n, h, wd, c = x.shape
    k = w.shape[0]
    ho, wo = (h - 1) // stride + 1, (wd - 1) // stride + 1
    X = torch.from_numpy(x.view(np.int16)).to(DEV)
    Wt = torch.from_numpy(w.view(np.int16)).to(DEV)
    Y = torch.zeros((n, ho, wo, k), dtype=torch.float32 if out_f32 else torch.int16, device=DEV)
    rc = mgb.mgb_conv3x3_enqueue(None, P(X), P(Wt), P(Y), n, h, wd, c, k, stride, 1 if out_f32 else 0)
    assert rc == 0, mgb.mgb_last_error()
    sync()
    y = Y.cpu().numpy()
    return y if out_f32 else y.view(np.uint16)


def _conv_inputs(seed, n, h, wd, c, k, sigma=0.2):
    x = W.f32_to_bf16_bits(W.uniform01(seed, n * h * wd * c).reshape(n, h, wd, c))
    w = W.f32_to_bf16_bits(W.normal(seed + 1, k * 9 * c, sigma=sigma).reshape(k, 3, 3, c))
    return x, w


@pytest.mark.parametrize("n,h,wd,c,k,stride", [
    (1, 8, 8, 3, 32, 1), (2, 13, 11, 3, 32, 2), (1, 16, 16, 8, 64, 1), (1, 17, 9, 32, 64, 2),
    (3, 12, 12, 64, 128, 1), (1, 26, 26, 40, 200, 2), (2, 7, 7, 128, 256, 1), (1, 5, 6, 5, 7, 1),
    (1, 1, 1, 8, 8, 1), (1, 40, 40, 16, 48, 2),
    # 3-channel first layer: several workgroups with a ragged tail, rows shorter and longer than a
    # workgroup's 256 pixels, two images, 64 channels
    (1, 40, 37, 3, 32, 1), (2, 9, 300, 3, 64, 1), (1, 3, 3, 3, 8, 1),
    # DMA ring, 64 x 64 tiles: ragged pixels and channels, c_in = 32 (one tile per tap) and 96
    (1, 1, 1, 32, 8, 1), (2, 9, 7, 96, 72, 2), (1, 20, 20, 256, 512, 1),
    # 64 x 64 tiles with the depth split over four waves (c_in % 64 == 0): odd and even tile counts
    (1, 1, 1, 64, 8, 1), (2, 9, 7, 192, 72, 2), (1, 13, 13, 512, 520, 1), (2, 31, 29, 64, 136, 1),
    # DMA ring, 128 x 128 and 256 x 64 tiles (at least 256 workgroups), stride 1 and 2, ragged tails
    (2, 130, 127, 32, 136, 1), (3, 150, 151, 32, 64, 1), (5, 141, 150, 64, 40, 2),
    # the same tiles fed by operand tiles of depth 64 (c_in % 64 == 0): 128 x 128, 256 x 64 at stride 1 and 2
    (2, 130, 127, 64, 136, 1), (3, 150, 151, 128, 64, 1), (13, 141, 150, 64, 40, 2),
    # stride 1 with the input patch in LDS: whole small images as tiles (idle pixel slots), three channel
    # blocks, ragged channels; 8 output channels (weight rows clamped)
    (70, 12, 13, 192, 72, 1), (4, 100, 90, 64, 8, 1),
    # stride 2 from 32 channels with the filter and the patch in LDS: ragged tiles, 64 and 40 output channels
    (5, 150, 151, 32, 64, 2), (6, 141, 150, 32, 40, 2)])
def test_conv_layer_fp32_and_bf16_outputs(n, h, wd, c, k, stride):
    x, w = _conv_inputs(n * 100 + c, n, h, wd, c, k)
    ref = oracle.conv3x3_relu(x, w, stride)
    got32 = run_conv(x, w, stride, True)
    assert got32.shape == ref.shape
    assert frobenius_rel(got32, ref) <= 1e-2 and frobenius_rel(got32, ref) <= 1e-5
    assert (got32 >= 0).all() and (ref == 0).any()                   # ReLU active
    got16 = run_conv(x, w, stride, False)
    want16 = oracle.round_bf16(ref)
    assert frobenius_rel(W.bf16_bits_to_f32(got16), ref) <= 1e-2
    # the rounding decision is taken from an fp32 value on both sides: at most one bf16 step apart,
    # and only where the fp32 accumulations straddle a rounding boundary.  A sum that cancels to
    # nearly zero keeps the absolute error of its terms (fp32 accumulation: a few 2^-24 of
    # sum |x||w|), which there is many steps of the tiny result: such entries are held to that
    # absolute bound instead.
    diff = np.abs(got16.astype(np.int32) - want16.astype(np.int32))
    mag = oracle.conv3x3_relu(x, W.f32_to_bf16_bits(np.abs(W.bf16_bits_to_f32(w))), stride)   # sum |x||w| (x >= 0)
    far = diff > 1
    assert (np.abs(W.bf16_bits_to_f32(got16).astype(np.float64) - ref)[far] <= 1e-5 * mag[far]).all()
    assert far.mean() <= 1e-3 and (diff != 0).mean() <= 0.01


def _layer_structs(layers):
    arr = (mgb.mgb_conv_layer * len(layers))()
    for i, L in enumerate(layers):
        arr[i] = mgb.mgb_conv_layer(L["c_in"], L["c_out"], L["stride"])
    return arr


def run_cnn(xb, weights, layers, batch, h, wd):
    arr = _layer_structs(layers)
    mem, act, ob = C.c_uint64(), C.c_uint64(), C.c_uint64()
    g, b = mgb.mgb_dim3(), mgb.mgb_dim3()
    assert mgb.mgb_cnn_probe(arr, len(layers), batch, h, wd, C.byref(mem), C.byref(act), C.byref(ob),
                             C.byref(g), C.byref(b)) == 0
    X = torch.from_numpy(xb.view(np.int16)).to(DEV)
    Wd = [torch.from_numpy(w.view(np.int16)).to(DEV) for w in weights]
    ptrs = (C.c_void_p * len(Wd))(*[t.data_ptr() for t in Wd])
    a0 = torch.zeros(max(1, act.value // 2), dtype=torch.int16, device=DEV)
    a1 = torch.zeros(max(1, act.value // 2), dtype=torch.int16, device=DEV)
    out = torch.zeros(ob.value // 4, dtype=torch.float32, device=DEV)
    total = X.numel() * 2 + sum(t.numel() * 2 for t in Wd) + 2 * act.value + ob.value
    assert mem.value == total                                       # footprint = sum of allocations
    rc = mgb.mgb_cnn_enqueue(None, arr, len(layers), P(X), ptrs, P(a0), P(a1), P(out), batch, h, wd)
    assert rc == 0, mgb.mgb_last_error()
    sync()
    L = layers[-1]
    return out.cpu().numpy().reshape(batch, L["h_out"], L["w_out"], L["c_out"]), mem.value, g, b


def test_cnn_ten_layer_chain_reduced_image():
    h = wd = 104
    layers = W.cnn_layers(h, wd)
    weights = W.cnn_weights(31, layers, sigma=0.02)
    xb = W.cnn_input(31, 2, h, wd)
    got, mem, g, b = run_cnn(xb, weights, layers, 2, h, wd)
    ref = oracle.cnn_forward(xb, weights, [L["stride"] for L in layers])
    assert got.shape == ref.shape == (2, 4, 4, 512)
    assert np.linalg.norm(ref) > 0
    assert frobenius_rel(got, ref) <= 1e-2
    # geometry of the task = the launch with the most threads: the last layer, 8 tiles of 64 x 64
    # (2*4*4 pixels x 512 channels) whose depth is split over 16 workgroups of 256 threads each
    # (the first layer has 2*104*104 / 256 -> 85 -> 88 workgroups)
    assert (g.x, b.x) == (128, 256)


def test_first_two_layers_in_one_kernel_match_the_layers_run_apart():
    # 3 -> 32 channels at stride 1, then 32 -> 64 (and 40) at stride 2: inside a chain the first layer is
    # computed by the second layer's kernel from the raw pixels under each patch.  Ragged tiles at
    # the right and bottom edges; 6 images x 48 tiles = 288 workgroups.
    batch, h, wd = 6, 150, 151
    for k2 in (64, 40):
        layers = [dict(c_in=3, c_out=32, stride=1, h_in=h, w_in=wd, h_out=h, w_out=wd),
                  dict(c_in=32, c_out=k2, stride=2, h_in=h, w_in=wd, h_out=75, w_out=76)]
        weights = W.cnn_weights(41 + k2, layers, sigma=0.2)
        xb = W.cnn_input(41, batch, h, wd)
        got, mem, g, b = run_cnn(xb, weights, layers, batch, h, wd)
        assert (g.x, b.x) == (288, 256)                              # the one launch of the chain
        # the same two layers through the single-layer entry point: the first layer's own kernel writes
        # its bf16 output, the second reads it back.  Same arithmetic in the same order: the same bits.
        y0 = run_conv(xb, weights[0], 1, False)
        apart = run_conv(y0, weights[1], 2, True)
        assert np.array_equal(got, apart)
        ref = oracle.cnn_forward(xb, weights, [1, 2])
        assert (ref == 0).any() and np.linalg.norm(ref) > 0
        assert frobenius_rel(got, ref) <= 1e-2 and frobenius_rel(got, ref) <= 1e-5


def test_chain_whose_buffers_are_not_16_byte_aligned_runs_its_first_two_layers_apart():
    # the same two layers, but the second layer's filter and both ping-pong buffers start 2 bytes off
    # a 16-byte boundary: the kernel that takes both layers cannot be used, each layer falls back to
    # a kernel without alignment needs, and the chain still matches the checker
    batch, h, wd = 6, 150, 151
    layers = [dict(c_in=3, c_out=32, stride=1, h_in=h, w_in=wd, h_out=h, w_out=wd),
              dict(c_in=32, c_out=64, stride=2, h_in=h, w_in=wd, h_out=75, w_out=76),
              dict(c_in=64, c_out=16, stride=2, h_in=75, w_in=76, h_out=38, w_out=38)]
    weights = W.cnn_weights(77, layers, sigma=0.2)
    xb = W.cnn_input(77, batch, h, wd)
    arr = _layer_structs(layers)
    mem, act, ob = C.c_uint64(), C.c_uint64(), C.c_uint64()
    g, b = mgb.mgb_dim3(), mgb.mgb_dim3()
    assert mgb.mgb_cnn_probe(arr, 3, batch, h, wd, C.byref(mem), C.byref(act), C.byref(ob), C.byref(g), C.byref(b)) == 0
    X = torch.from_numpy(xb.view(np.int16)).to(DEV)
    Wd = [torch.zeros(w.size + 8, dtype=torch.int16, device=DEV) for w in weights]
    for t, w in zip(Wd, weights):
        t[1:1 + w.size] = torch.from_numpy(w.view(np.int16).ravel()).to(DEV)
    ptrs = (C.c_void_p * 3)(*[t.data_ptr() + 2 for t in Wd])
    a0 = torch.zeros(act.value // 2 + 8, dtype=torch.int16, device=DEV)
    a1 = torch.zeros(act.value // 2 + 8, dtype=torch.int16, device=DEV)
    out = torch.zeros(ob.value // 4, dtype=torch.float32, device=DEV)
    rc = mgb.mgb_cnn_enqueue(None, arr, 3, P(X), ptrs, C.c_void_p(a0.data_ptr() + 2), C.c_void_p(a1.data_ptr() + 2), P(out), batch, h, wd)
    assert rc == 0, mgb.mgb_last_error()
    sync()
    got = out.cpu().numpy().reshape(batch, 38, 38, 16)
    ref = oracle.cnn_forward(xb, weights, [1, 2, 2])
    assert np.linalg.norm(ref) > 0 and frobenius_rel(got, ref) <= 1e-2


def test_cnn_full_size_layers_sampled():
    # 416x416 input, batch 1: every layer of the real net is checked on sampled output pixels,
    # each recomputed by the checker from the 3x3xC patch of that layer's (GPU-produced) input
    h = wd = 416
    layers = W.cnn_layers(h, wd)
    weights = W.cnn_weights(8, layers)
    act = W.cnn_input(8, 1, h, wd)
    rng = np.random.default_rng(0)
    for li, L in enumerate(layers):
        last = li + 1 == len(layers)
        y = run_conv(act, weights[li], L["stride"], last)
        ho, wo = L["h_out"], L["w_out"]
        assert y.shape == (1, ho, wo, L["c_out"])
        pts = [(0, 0), (0, wo - 1), (ho - 1, 0), (ho - 1, wo - 1)] + \
              [(int(rng.integers(0, ho)), int(rng.integers(0, wo))) for _ in range(12)]
        for oh, ow in pts:
            patch = np.zeros((1, 3, 3, L["c_in"]), dtype=np.uint16)
            for r in range(3):
                for s in range(3):
                    ih, iw = oh * L["stride"] - 1 + r, ow * L["stride"] - 1 + s
                    if 0 <= ih < L["h_in"] and 0 <= iw < L["w_in"]:
                        patch[0, r, s] = act[0, ih, iw]
            want = oracle.conv3x3_relu(patch, weights[li], 1)[0, 1, 1]
            have = y[0, oh, ow] if last else W.bf16_bits_to_f32(y[0, oh, ow])
            assert np.linalg.norm(have - want) <= 1e-2 * max(np.linalg.norm(want), 1e-6), (li, oh, ow)
        act = y


def test_conv_rejects_bad_arguments():
    t = torch.zeros(1024, dtype=torch.int16, device=DEV)
    assert mgb.mgb_conv3x3_enqueue(None, P(t), P(t), P(t), 1, 4, 4, 8, 8, 3, 0) == mgb.MGB_E_UNSUPPORTED
    assert mgb.mgb_conv3x3_enqueue(None, None, P(t), P(t), 1, 4, 4, 8, 8, 1, 0) == mgb.MGB_E_INVAL
    assert mgb.mgb_conv3x3_enqueue(None, P(t), P(t), P(t), 0, 4, 4, 8, 8, 1, 0) == mgb.MGB_E_UNSUPPORTED


# ------------------------------------------------------------------ BFS
def run_bfs(rp, ci, source=0, directed=False):
    n = rp.size - 1
    RP = torch.from_numpy(rp).to(DEV)
    CI = torch.from_numpy(ci if ci.size else np.zeros(1, np.int32)).to(DEV)
    lev = torch.full((n,), -7, dtype=torch.int32, device=DEV)
    work = torch.zeros(mgb.mgb_bfs_work_bytes(n), dtype=torch.uint8, device=DEV)
    depth = u32(0)
    st = torch.cuda.current_stream().cuda_stream
    fn = mgb.mgb_bfs_directed_enqueue if directed else mgb.mgb_bfs_enqueue
    rc = fn(C.c_void_p(st), P(RP), P(CI), n, source, P(lev), P(work), C.byref(depth))
    assert rc == 0, mgb.mgb_last_error()
    sync()
    return lev.cpu().numpy(), depth.value


def _csr(n, edges):
    e = np.array(edges, dtype=np.int64).reshape(-1, 2)
    s = np.concatenate([e[:, 0], e[:, 1]])
    d = np.concatenate([e[:, 1], e[:, 0]])
    order = np.lexsort((d, s))
    s, d = s[order], d[order]
    rp = np.zeros(n + 1, dtype=np.int32)
    np.cumsum(np.bincount(s, minlength=n), out=rp[1:])
    return rp, d.astype(np.int32)


@pytest.mark.parametrize("seed,n,deg", [(1, 1000, 3), (2, 5000, 1), (3, 1 << 16, 8), (4, 70000, 16),
                                        (5, 100, 30), (6, 1 << 18, 32),
                                        # more than 2^20 vertices: the frontier bitmap stays in memory;
                                        # a span of 256 vertices that ends ragged; 37 levels in three batches
                                        ((1 << 20) + 777, (1 << 20) + 777, 6), (8, 300001, 2.2)])
def test_bfs_random_graphs_bit_exact(seed, n, deg):
    rp, ci = W.er_graph_csr(seed, n, deg)
    got, depth = run_bfs(rp, ci)
    want = oracle.bfs(rp, ci, 0)
    assert np.array_equal(got, want)
    assert depth == want.max() + 1


@pytest.mark.parametrize("seed,n,deg", [(1, 1000, 3), (2, 40000, 2), (3, 200000, 8), (4, 5000, 0.7)])
def test_bfs_directed_graphs_bit_exact(seed, n, deg):
    # arcs stored once: reachability is one-way, and expanding a level from the unvisited side
    # (which reads stored edges as in-edges) would be wrong here
    rp, ci = W.er_digraph_csr(seed, n, deg)
    got, depth = run_bfs(rp, ci, source=seed % n, directed=True)
    ref = oracle.bfs(rp, ci, seed % n)
    assert np.array_equal(got, ref)
    assert depth == ref.max() + 1
    # a one-way chain: only the vertices downstream of the source are reached
    m = 300
    rp = np.arange(m + 1, dtype=np.int32)
    rp[-1] = m - 1
    ci = np.arange(1, m, dtype=np.int32)
    got, depth = run_bfs(rp, ci, source=100, directed=True)
    want = np.where(np.arange(m) >= 100, np.arange(m) - 100, -1).astype(np.int32)
    assert np.array_equal(got, want) and depth == 200


def test_bfs_degenerate_graphs():
    n = 300                                                         # path: 300 levels, many batches
    rp, ci = _csr(n, [(i, i + 1) for i in range(n - 1)])
    got, depth = run_bfs(rp, ci, 0)
    assert np.array_equal(got, np.arange(n)) and depth == n
    got, _ = run_bfs(rp, ci, 150)
    assert np.array_equal(got, np.abs(np.arange(n) - 150))
    rp, ci = _csr(5000, [(0, i) for i in range(1, 5000)])           # star: one huge adjacency list
    got, depth = run_bfs(rp, ci, 0)
    assert np.array_equal(got, np.r_[0, np.ones(4999, dtype=np.int32)]) and depth == 2
    got, _ = run_bfs(rp, ci, 17)
    assert got[0] == 1 and got[17] == 0 and got[18] == 2
    rp = np.zeros(11, dtype=np.int32)                               # no edges at all
    got, depth = run_bfs(rp, np.zeros(0, np.int32), 4)
    assert list(got) == [-1] * 4 + [0] + [-1] * 5 and depth == 1
    rp, ci = _csr(1, [])                                            # single vertex
    got, depth = run_bfs(rp, ci, 0)
    assert list(got) == [0] and depth == 1
    for n in (16, 17, 18, 32, 33, 34, 56, 57, 58):                  # depths around the batch sizes (8, then 16, then 32)
        rp, ci = _csr(n, [(i, i + 1) for i in range(n - 1)])
        got, depth = run_bfs(rp, ci, 0)
        assert np.array_equal(got, np.arange(n)) and depth == n
    # a hub as the source and as the second level; a wide second level whose vertices have one edge each
    rp, ci = _csr(20000, [(0, i) for i in range(1, 20000)])
    got, depth = run_bfs(rp, ci, 0)
    assert np.array_equal(got, np.r_[0, np.ones(19999, dtype=np.int32)]) and depth == 2
    got, depth = run_bfs(rp, ci, 9)
    assert got[0] == 1 and got[9] == 0 and (np.delete(got, [0, 9]) == 2).all() and depth == 3
    edges = [(0, i) for i in range(1, 3001)] + [(i, i + 3000) for i in range(1, 3001)] + [(6000, 6001)]
    rp, ci = _csr(6002, edges)
    got, depth = run_bfs(rp, ci, 0)
    want = oracle.bfs(rp, ci, 0)
    assert np.array_equal(got, want) and depth == want.max() + 1 == 4
    got, depth = run_bfs(rp, ci, 6001)
    want = oracle.bfs(rp, ci, 6001)
    assert np.array_equal(got, want) and depth == want.max() + 1


def test_bfs_full_size_mix16_task():
    rp, ci = W.er_graph_csr(2020, 1 << 20, 16)
    got, depth = run_bfs(rp, ci)
    want = oracle.bfs(rp, ci, 0)
    assert np.array_equal(got, want) and depth == want.max() + 1


def test_bfs_rejects_bad_arguments():
    t = torch.zeros(4096, dtype=torch.int32, device=DEV)
    assert mgb.mgb_bfs_enqueue(None, P(t), P(t), 4, 4, P(t), P(t), None) == mgb.MGB_E_INVAL   # source >= n
    assert mgb.mgb_bfs_enqueue(None, P(t), P(t), 0, 0, P(t), P(t), None) == mgb.MGB_E_INVAL
    assert mgb.mgb_bfs_enqueue(None, P(t), P(t), 4, 0, P(t), None, None) == mgb.MGB_E_INVAL
