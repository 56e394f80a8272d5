"""Parity on seeded random shapes: every kernel family against the CPU checker on shapes nobody
chose by hand (ragged tails, every tile variant, odd depths), to the same tolerances as the
hand-picked cases in test_gpu_kernels.py."""
import numpy as np
import pytest

import oracle
import workloads as W
from helpers import frobenius_rel
import test_gpu_kernels as K

pytestmark = pytest.mark.gpu


def _r(rng, lo, hi):
    return int(rng.integers(lo, hi + 1))


@pytest.mark.parametrize("seed", [1, 2])
def test_random_gemm_shapes(seed):
    rng = np.random.default_rng(seed)
    for i in range(16):
        m, n, k = _r(rng, 1, 900), _r(rng, 1, 900), _r(rng, 1, 700)
        if i % 2 == 0:                                    # the DMA-ring kernels' shapes
            k, n = 16 * _r(rng, 1, 40), 4 * _r(rng, 1, 225)
        if i % 8 == 0:                                    # enough 128 x 128 tiles for that variant
            m, n = _r(rng, 1300, 1700), 4 * _r(rng, 330, 420)
        a, b = W.gemm_operands_f32(1000 * seed + i, m, n, k)
        got = K.run_gemm_f32(a, b)
        ref, den = oracle.gemm_f32(a, b), oracle.gemm_abs_f32(a, b)
        assert (np.abs(got.astype(np.float64) - ref) / den).max() <= 1e-4, ("f32", m, n, k)
    for i in range(16):
        m, n, k = _r(rng, 1, 900), _r(rng, 1, 900), _r(rng, 1, 700)
        if i % 2 == 0:
            k, n = 32 * _r(rng, 1, 20), 8 * _r(rng, 1, 110)
        if i % 8 == 0:                                    # at least 128 tiles of 256 x 256
            m, n = _r(rng, 2700, 3000), 8 * _r(rng, 352, 380)
        ab, bb = W.gemm_operands_bf16(2000 * seed + i, m, n, k)
        assert frobenius_rel(K.run_gemm_bf16(ab, bb), oracle.gemm_bf16(ab, bb)) <= 1e-5, ("bf16", m, n, k)


@pytest.mark.parametrize("seed", [3])
def test_random_conv_layers_and_chains(seed):
    rng = np.random.default_rng(seed)
    chans = [3, 8, 32, 64, 96, 128, 192, 5, 40]
    outs = [8, 32, 64, 72, 128, 136, 7, 200]
    for i in range(16):
        n, h, w, st = _r(rng, 1, 3), _r(rng, 1, 40), _r(rng, 1, 40), _r(rng, 1, 2)
        c, k = chans[_r(rng, 0, 8)], outs[_r(rng, 0, 7)]
        if i % 5 == 0:
            h, w = _r(rng, 100, 160), _r(rng, 100, 160)
        x, wt = K._conv_inputs(3000 + i, n, h, w, c, k)
        ref = oracle.conv3x3_relu(x, wt, st)
        assert frobenius_rel(K.run_conv(x, wt, st, True), ref) <= 1e-5, (n, h, w, c, k, st)
        assert frobenius_rel(W.bf16_bits_to_f32(K.run_conv(x, wt, st, False)), ref) <= 1e-2, (n, h, w, c, k, st)
    widths = [8, 32, 64, 128, 256, 512, 40, 96]
    for i in range(8):
        nl, b, h, w = _r(rng, 1, 6), _r(rng, 1, 3), _r(rng, 6, 60), _r(rng, 6, 60)
        c = 3 if i % 2 == 0 else widths[_r(rng, 0, 7)]
        layers, hh, ww = [], h, w
        for _ in range(nl):
            co, st = widths[_r(rng, 0, 7)], _r(rng, 1, 2)
            ho, wo = (hh - 1) // st + 1, (ww - 1) // st + 1
            layers.append(dict(c_in=c, c_out=co, stride=st, h_in=hh, w_in=ww, h_out=ho, w_out=wo))
            c, hh, ww = co, ho, wo
        weights = W.cnn_weights(4000 + i, layers, sigma=0.05)
        xb = W.cnn_input(4000 + i, b, h, w, layers[0]["c_in"])
        got, mem, g, blk = K.run_cnn(xb, weights, layers, b, h, w)
        ref = oracle.cnn_forward(xb, weights, [L["stride"] for L in layers])
        if np.linalg.norm(ref) > 0:
            assert frobenius_rel(got, ref) <= 1e-2, [(L["c_in"], L["c_out"], L["stride"]) for L in layers]
        else:
            assert np.abs(got).max() == 0.0


@pytest.mark.parametrize("seed", [4])
def test_random_jacobi_and_bfs(seed):
    rng = np.random.default_rng(seed)
    for i in range(12):
        n, it = _r(rng, 3, 1500), _r(rng, 1, 13)
        u = W.jacobi_field(5000 + i, n)
        assert np.array_equal(K.run_jacobi(u, it), oracle.jacobi_f32(u, it)), (n, it)
    for i in range(10):
        n, d = _r(rng, 2, 300000), float(rng.uniform(0.5, 20))
        rp, ci = W.er_graph_csr(6000 + i, n, d)
        got, depth = K.run_bfs(rp, ci)
        want = oracle.bfs(rp, ci, 0)
        assert np.array_equal(got, want) and depth == want.max() + 1, (n, d)


def _sym_csr(n, s, d):
    s2, d2 = np.concatenate([s, d]), np.concatenate([d, s])
    order = np.lexsort((d2, s2))
    s2, d2 = s2[order], d2[order]
    rp = np.zeros(n + 1, dtype=np.int32)
    np.cumsum(np.bincount(s2, minlength=n), out=rp[1:])
    return rp, d2.astype(np.int32)


@pytest.mark.parametrize("seed", [31])
def test_random_skewed_graphs(seed):
    """Degree distributions far from the benchmark's: a few rows of thousands of entries (spans of the
    bottom-up scan whose edges do not fit its bit array), blocks of isolated vertices between dense
    ones (zero-length rows inside a span), more than 2^20 vertices (frontier bitmap in memory), any source."""
    rng = np.random.default_rng(seed)
    for i in range(9):
        kind = i % 3
        if kind == 0:
            n = _r(rng, 1000, 600000)
            m = int(n * rng.uniform(2, 12))
            s = (n * rng.random(m) ** 3).astype(np.int64)
            d = rng.integers(0, n, m)
            src = _r(rng, 0, n - 1)
        elif kind == 1:
            n = _r(rng, 1000, 500000)
            m = int(n * rng.uniform(4, 20))
            ids = np.flatnonzero(rng.random(n) < 0.5)
            s, d = ids[rng.integers(0, ids.size, m)], ids[rng.integers(0, ids.size, m)]
            src = int(ids[0])
        else:
            n = _r(rng, 1 << 20, 2 << 20)
            m = int(n * rng.uniform(1.0, 5.0))
            s, d = rng.integers(0, n, m), rng.integers(0, n, m)
            src = _r(rng, 0, n - 1)
        keep = s != d
        rp, ci = _sym_csr(n, s[keep], d[keep])
        got, depth = K.run_bfs(rp, ci, src)
        want = oracle.bfs(rp, ci, src)
        assert np.array_equal(got, want) and depth == want.max() + 1, (kind, n, m, src)
