"""Pins for the CPU checker's task kernels: closed forms, library routines,
invariants and brute force -- nothing here compares the checker with itself."""
import numpy as np
import pytest
import scipy.ndimage
import scipy.signal
import scipy.sparse as sp
import scipy.sparse.csgraph as csgraph

import oracle
import workloads as W


# ------------------------------------------------------------------ Jacobi
def test_jacobi_constant_field_is_fixed_point():
    # (c+c)+(c+c) and the scaling by 1/4 are exact: interior = ring = c stays c, bit for bit
    for c in (0.0, 1.0, 0.3, -7.25):
        u = np.full((9, 9), c, dtype=np.float32)
        assert np.array_equal(oracle.jacobi_f32(u, 7), u)
        assert np.array_equal(oracle.jacobi_f64(u, 7), u.astype(np.float64))


@pytest.mark.parametrize("n,p,q,k", [(17, 1, 1, 10), (33, 2, 3, 6), (20, 5, 1, 9)])
def test_jacobi_eigenmode_closed_form(n, p, q, k):
    # sin(pi p i/(n-1)) sin(pi q j/(n-1)) vanishes on the ring and is an eigenvector of the
    # sweep with eigenvalue (cos(pi p/(n-1)) + cos(pi q/(n-1)))/2
    i = np.arange(n)
    u0 = np.outer(np.sin(np.pi * p * i / (n - 1)), np.sin(np.pi * q * i / (n - 1)))
    u0[0, :] = u0[-1, :] = 0.0
    u0[:, 0] = u0[:, -1] = 0.0
    lam = 0.5 * (np.cos(np.pi * p / (n - 1)) + np.cos(np.pi * q / (n - 1)))
    got = oracle.jacobi_f64(u0, k)
    assert np.abs(got - lam ** k * u0).max() < 1e-13
    got32 = oracle.jacobi_f32(u0.astype(np.float32), k)
    assert np.abs(got32 - lam ** k * u0).max() < 5e-6


def test_jacobi_equals_library_convolution():
    # one sweep on the interior is a correlation with the 5-point kernel (library routine)
    rng = np.random.default_rng(3)
    n = 12
    u = rng.random((n, n))
    u[0, :] = u[-1, :] = 0.0
    u[:, 0] = u[:, -1] = 0.0
    kern = np.array([[0, .25, 0], [.25, 0, .25], [0, .25, 0]])
    cur = u.copy()
    for _ in range(5):
        nxt = scipy.ndimage.correlate(cur, kern, mode="constant")
        nxt[0, :] = nxt[-1, :] = 0.0
        nxt[:, 0] = nxt[:, -1] = 0.0
        cur = nxt
    assert np.abs(oracle.jacobi_f64(u, 5) - cur).max() < 1e-14


def test_jacobi_nonzero_ring_is_kept_and_used():
    # ring values stay fixed and feed their neighbours: 3x3 grid, single interior cell
    u = np.array([[1, 2, 3], [4, 100, 6], [7, 8, 9]], dtype=np.float64)
    got = oracle.jacobi_f64(u, 1)
    want = u.copy()
    want[1, 1] = (2 + 8 + 4 + 6) / 4.0
    assert np.array_equal(got, want)
    assert np.array_equal(oracle.jacobi_f64(u, 2), want)   # ring fixed => same value again
    # asymmetric 4x4: distinguishes north/south/west/east and row/column order
    u = np.arange(16, dtype=np.float64).reshape(4, 4) ** 2
    got = oracle.jacobi_f64(u, 1)
    for i in (1, 2):
        for j in (1, 2):
            assert got[i, j] == (u[i - 1, j] + u[i + 1, j] + u[i, j - 1] + u[i, j + 1]) / 4.0


def test_jacobi_maximum_principle_and_decay():
    u = W.jacobi_field(11, 24)
    prev = u.astype(np.float64)
    for k in range(1, 6):
        cur = oracle.jacobi_f64(u, k)
        assert cur.max() <= prev.max() + 1e-15 and cur.min() >= 0.0
        prev = cur
    assert oracle.jacobi_f64(u, 4000).max() < 1e-6      # zero ring => relaxes to zero


def test_jacobi_f32_matches_f64_to_rounding():
    u = W.jacobi_field(5, 40)
    a = oracle.jacobi_f32(u, 50).astype(np.float64)
    b = oracle.jacobi_f64(u, 50)
    inner = b[1:-1, 1:-1]
    assert (np.abs(a - b)[1:-1, 1:-1] / inner).max() < 1e-5
    assert np.all(a[0, :] == 0) and np.all(a[:, -1] == 0)


# ------------------------------------------------------------------ GEMM
def test_gemm_identity_permutation_rank1():
    rng = np.random.default_rng(0)
    a = rng.standard_normal((7, 5)).astype(np.float32)
    assert np.array_equal(oracle.gemm_f32(a, np.eye(5, dtype=np.float32)), a.astype(np.float64))
    perm = np.eye(5, dtype=np.float32)[[2, 0, 4, 1, 3]]
    # (A P)[i][j] = A[i][sigma(j)] for P[sigma(j)][j] = 1
    assert np.array_equal(oracle.gemm_f32(a, perm.T.copy()), a[:, [2, 0, 4, 1, 3]].astype(np.float64))
    u = rng.standard_normal((6, 1)).astype(np.float32)
    v = rng.standard_normal((1, 4)).astype(np.float32)
    assert np.array_equal(oracle.gemm_f32(u, v), u.astype(np.float64) * v.astype(np.float64))


@pytest.mark.parametrize("m,n,k", [(3, 5, 7), (16, 9, 33), (40, 41, 42)])
def test_gemm_matches_library_matmul(m, n, k):
    a, b = W.gemm_operands_f32(9, m, n, k)
    ref = a.astype(np.float64) @ b.astype(np.float64)
    got = oracle.gemm_f32(a, b)
    assert np.abs(got - ref).max() <= 1e-13 * np.abs(ref).max() + 1e-13
    den = oracle.gemm_abs_f32(a, b)
    assert np.abs(den - np.abs(a).astype(np.float64) @ np.abs(b).astype(np.float64)).max() < 1e-12
    rows = np.array([0, m - 1, m // 2], dtype=np.uint32)
    cols = np.array([n - 1, 0, n // 2], dtype=np.uint32)
    e, ea = oracle.gemm_f32_entries(a, b, rows, cols)
    assert np.allclose(e, ref[rows, cols], rtol=0, atol=1e-12)
    assert np.allclose(ea, den[rows, cols], rtol=0, atol=1e-12)


def test_gemm_bf16_decodes_bits_and_matches_library():
    # bf16 bit patterns with known values: 0x3F80 = 1, 0xC000 = -2, 0x3F00 = 0.5, 0x4049 = 3.140625
    a = np.array([[0x3F80, 0xC000], [0x3F00, 0x4049]], dtype=np.uint16)
    b = np.array([[0x3F80, 0x3F00], [0xC000, 0x3F80]], dtype=np.uint16)
    want = np.array([[1 * 1 + -2 * -2, 1 * .5 + -2 * 1], [.5 * 1 + 3.140625 * -2, .25 + 3.140625]])
    assert np.array_equal(oracle.gemm_bf16(a, b), want)
    ab, bb = W.gemm_operands_bf16(4, 11, 13, 17)
    ref = W.bf16_bits_to_f32(ab).astype(np.float64) @ W.bf16_bits_to_f32(bb).astype(np.float64)
    got = oracle.gemm_bf16(ab, bb)
    assert np.abs(got - ref).max() < 1e-12
    rows = np.array([10, 0], dtype=np.uint32)
    cols = np.array([12, 3], dtype=np.uint32)
    assert np.allclose(oracle.gemm_bf16_entries(ab, bb, rows, cols), ref[rows, cols], atol=1e-12)


def test_round_bf16_nearest_even():
    # 1 + 2^-8 is a tie between 1.0 (even mantissa) and 1 + 2^-7 -> 1.0; 1 + 3*2^-8 ties up to 1+2^-6
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -2.5, 0.0])
    got = oracle.round_bf16(x)
    assert list(got) == [0x3F80, 0x3F80, 0x3F82, 0x3F81, 0xC020, 0x0000]
    # agrees with the input generator's converter on random data (two separate implementations)
    r = np.random.default_rng(1).standard_normal(1000).astype(np.float32)
    assert np.array_equal(oracle.round_bf16(r.astype(np.float64)), W.f32_to_bf16_bits(r))


# ------------------------------------------------------------------ conv
def _bits(x):
    return W.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def _val(bits):
    return W.bf16_bits_to_f32(bits).astype(np.float64)


@pytest.mark.parametrize("stride", [1, 2])
def test_conv_centre_tap_is_a_gemm(stride):
    rng = np.random.default_rng(5)
    x = _bits(rng.standard_normal((2, 6, 7, 5)))
    w = np.zeros((4, 3, 3, 5), dtype=np.float32)
    w[:, 1, 1, :] = rng.standard_normal((4, 5))
    w = _bits(w)
    y = oracle.conv3x3_relu(x, w, stride)
    want = np.maximum(0.0, np.einsum("nhwc,kc->nhwk", _val(x)[:, ::stride, ::stride, :], _val(w)[:, 1, 1, :]))
    assert y.shape == want.shape
    assert np.abs(y - want).max() < 1e-12


@pytest.mark.parametrize("h,wd", [(5, 5), (6, 9)])
def test_conv_all_ones_counts_taps_inside(h, wd):
    c = 3
    x = _bits(np.ones((1, h, wd, c)))
    w = _bits(np.ones((2, 3, 3, c)))
    y = oracle.conv3x3_relu(x, w, 1)
    rows = np.array([2] + [3] * (h - 2) + [2])
    cols = np.array([2] + [3] * (wd - 2) + [2])
    want = np.outer(rows, cols) * c            # taps inside the image x channels
    assert np.array_equal(y[0, :, :, 0], want) and np.array_equal(y[0, :, :, 1], want)
    y2 = oracle.conv3x3_relu(x, w, 2)
    assert y2.shape == (1, (h - 1) // 2 + 1, (wd - 1) // 2 + 1, 2)
    assert np.array_equal(y2[0, :, :, 0], want[::2, ::2])   # stride 2 = stride 1 at even positions


def test_conv_matches_library_correlation_and_relu():
    rng = np.random.default_rng(8)
    n, h, wd, c, k = 2, 7, 6, 3, 4
    x = _bits(rng.standard_normal((n, h, wd, c)))
    w = _bits(rng.standard_normal((k, 3, 3, c)))
    y = oracle.conv3x3_relu(x, w, 1)
    xv, wv = _val(x), _val(w)
    want = np.zeros((n, h, wd, k))
    for b in range(n):
        for kk in range(k):
            for cc in range(c):
                want[b, :, :, kk] += scipy.signal.correlate2d(xv[b, :, :, cc], wv[kk, :, :, cc], mode="same")
    assert (want < 0).any()
    assert np.abs(y - np.maximum(want, 0.0)).max() < 1e-12
    y2 = oracle.conv3x3_relu(x, w, 2)
    assert np.abs(y2 - np.maximum(want, 0.0)[:, ::2, ::2, :]).max() < 1e-12


def test_cnn_chain_rounds_between_layers():
    rng = np.random.default_rng(2)
    x = _bits(rng.random((1, 8, 8, 3)))
    w1 = _bits(rng.standard_normal((4, 3, 3, 3)) * 0.3)
    w2 = _bits(rng.standard_normal((5, 3, 3, 4)) * 0.3)
    y = oracle.cnn_forward(x, [w1, w2], [1, 2])
    mid = W.f32_to_bf16_bits(oracle.conv3x3_relu(x, w1, 1).astype(np.float32))
    want = oracle.conv3x3_relu(mid, w2, 2)
    assert y.shape == (1, 4, 4, 5) and np.array_equal(y, want)


def test_cnn_layer_table_matches_stated_shapes():
    L = W.cnn_layers()
    assert [l["c_out"] for l in L] == [32, 64, 64, 128, 128, 256, 256, 512, 512, 512]
    assert [l["stride"] for l in L] == [1, 2] * 5
    assert [l["h_out"] for l in L] == [416, 208, 208, 104, 104, 52, 52, 26, 26, 13]
    params = sum(l["c_out"] * 9 * l["c_in"] for l in L)
    assert abs(params - 7.06e6) < 0.01e6


# ------------------------------------------------------------------ BFS
def _csr(n, edges):
    e = np.array(edges, dtype=np.int64).reshape(-1, 2)
    s = np.concatenate([e[:, 0], e[:, 1]])
    d = np.concatenate([e[:, 1], e[:, 0]])
    order = np.lexsort((d, s))
    s, d = s[order], d[order]
    rp = np.zeros(n + 1, dtype=np.int32)
    np.cumsum(np.bincount(s, minlength=n), out=rp[1:])
    return rp, d.astype(np.int32)


def test_bfs_closed_form_graphs():
    n = 50
    rp, ci = _csr(n, [(i, i + 1) for i in range(n - 1)])
    assert np.array_equal(oracle.bfs(rp, ci, 0), np.arange(n))
    assert np.array_equal(oracle.bfs(rp, ci, 20), np.abs(np.arange(n) - 20))
    rp, ci = _csr(n, [(0, i) for i in range(1, n)])
    assert np.array_equal(oracle.bfs(rp, ci, 0), np.r_[0, np.ones(n - 1, dtype=int)])
    assert np.array_equal(oracle.bfs(rp, ci, 7)[[0, 7, 8]], [1, 0, 2])
    m = 127   # complete binary tree: level = floor(log2(v+1))
    rp, ci = _csr(m, [((v - 1) // 2, v) for v in range(1, m)])
    assert np.array_equal(oracle.bfs(rp, ci, 0), np.floor(np.log2(np.arange(m) + 1)).astype(int))
    r, c = 9, 13   # 2-D grid: Manhattan distance
    edges = [(i * c + j, i * c + j + 1) for i in range(r) for j in range(c - 1)]
    edges += [(i * c + j, (i + 1) * c + j) for i in range(r - 1) for j in range(c)]
    rp, ci = _csr(r * c, edges)
    ii, jj = np.divmod(np.arange(r * c), c)
    assert np.array_equal(oracle.bfs(rp, ci, 0), ii + jj)


def test_bfs_unreachable_and_isolated_source():
    rp, ci = _csr(6, [(0, 1), (1, 2), (3, 4)])
    assert list(oracle.bfs(rp, ci, 0)) == [0, 1, 2, -1, -1, -1]
    assert list(oracle.bfs(rp, ci, 5)) == [-1, -1, -1, -1, -1, 0]


@pytest.mark.parametrize("seed,n,deg", [(1, 300, 3), (2, 1000, 1), (3, 64, 6)])
def test_bfs_matches_library_shortest_path_and_floyd_warshall(seed, n, deg):
    rp, ci = W.er_graph_csr(seed, n, deg)
    lev = oracle.bfs(rp, ci, 0)
    g = sp.csr_matrix((np.ones(ci.size), ci, rp), shape=(n, n))
    dist = csgraph.shortest_path(g, method="D", unweighted=True, indices=0)
    want = np.where(np.isinf(dist), -1, dist).astype(np.int32)
    assert np.array_equal(lev, want)
    if n <= 64:
        fw = csgraph.floyd_warshall(g, unweighted=True)[0]
        assert np.array_equal(lev, np.where(np.isinf(fw), -1, fw).astype(np.int32))
    # structural invariants that hold for any correct level array
    src = np.repeat(np.arange(n), np.diff(rp))
    both = (lev[src] >= 0) & (lev[ci] >= 0)
    assert np.all(np.abs(lev[src][both] - lev[ci][both]) <= 1)
    assert np.all((lev[src] >= 0) == (lev[ci] >= 0))          # components are all-or-nothing
    ncomp, label = csgraph.connected_components(g, directed=False)
    assert np.array_equal(lev >= 0, label == label[0])


def test_er_generator_shape():
    rp, ci = W.er_graph_csr(7, 1 << 12, 16)
    n = 1 << 12
    assert rp[0] == 0 and rp[-1] == ci.size and ci.size <= n * 16
    assert ci.size > n * 16 * 0.99                              # few self-loops dropped
    src = np.repeat(np.arange(n), np.diff(rp))
    assert not np.any(src == ci)
    fwd = np.sort(src.astype(np.int64) * n + ci)
    bwd = np.sort(ci.astype(np.int64) * n + src)
    assert np.array_equal(fwd, bwd)                             # symmetric
    assert all(np.all(np.diff(ci[rp[v]:rp[v + 1]]) >= 0) for v in range(0, n, 97))
