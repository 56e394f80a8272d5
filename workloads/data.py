"""Synthetic task inputs with the shapes and value distributions of the task mixes."""
import numpy as np

from .rng import (raw64, uniform01, normal, f32_to_bf16_bits)


def jacobi_field(seed, n):
    """n x n float32 grid: interior U[0,1), outermost ring exactly zero."""
    u = uniform01(seed, n * n).reshape(n, n)
    u[0, :] = 0.0
    u[-1, :] = 0.0
    u[:, 0] = 0.0
    u[:, -1] = 0.0
    return u


def gemm_operands_f32(seed, m, n, k):
    """Row-major A (m x k) and B (k x n), entries N(0,1), float32."""
    a = normal(seed, m * k).reshape(m, k)
    b = normal(seed ^ 0xB, k * n).reshape(k, n)
    return a, b


def gemm_operands_bf16(seed, m, n, k):
    """Row-major A, B with N(0,1) entries rounded to bfloat16; uint16 bit patterns."""
    a, b = gemm_operands_f32(seed, m, n, k)
    return f32_to_bf16_bits(a), f32_to_bf16_bits(b)


def er_graph_csr(seed, n, mean_degree):
    """Undirected Erdos-Renyi-style multigraph G(n, m = n*mean_degree/2) as CSR.

    Edge endpoints are i.i.d. uniform vertices, self-loops are dropped,
    duplicate edges are kept, every edge is stored in both directions and each
    adjacency list is sorted.  Returns (row_ptr int32[n+1], col_idx int32[2m']).
    """
    m = int(n * mean_degree) // 2
    idx = np.arange(m, dtype=np.uint64)
    src = (raw64(seed, idx * np.uint64(2)) % np.uint64(n)).astype(np.int64)
    dst = (raw64(seed, idx * np.uint64(2) + np.uint64(1)) % np.uint64(n)).astype(np.int64)
    keep = src != dst
    src, dst = src[keep], dst[keep]
    s = np.concatenate([src, dst])
    d = np.concatenate([dst, src])
    key = s * np.int64(n) + d
    key.sort(kind="stable")
    s = key // n
    d = key - s * n
    counts = np.bincount(s, minlength=n)
    row_ptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(counts, out=row_ptr[1:])
    assert row_ptr[-1] < 2 ** 31
    return row_ptr.astype(np.int32), d.astype(np.int32)


def er_digraph_csr(seed, n, mean_out_degree):
    """Directed counterpart: n*mean_out_degree arcs with i.i.d. uniform endpoints, self-loops
    dropped, duplicates kept, each arc stored once (at its tail), adjacency lists sorted."""
    m = int(n * mean_out_degree)
    idx = np.arange(m, dtype=np.uint64)
    src = (raw64(seed, idx * np.uint64(2)) % np.uint64(n)).astype(np.int64)
    dst = (raw64(seed, idx * np.uint64(2) + np.uint64(1)) % np.uint64(n)).astype(np.int64)
    keep = src != dst
    key = src[keep] * np.int64(n) + dst[keep]
    key.sort(kind="stable")
    s = key // n
    d = key - s * n
    row_ptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.bincount(s, minlength=n), out=row_ptr[1:])
    assert row_ptr[-1] < 2 ** 31
    return row_ptr.astype(np.int32), d.astype(np.int32)


def cnn_layers(h=416, w=416, c_in=3):
    """Layer table of the 10-layer 3x3 conv+ReLU net: stride alternates 1,2 and
    the channel count doubles on stride-2 layers up to a cap of 512.
    Returns a list of dicts (c_in, c_out, stride, h_in, w_in, h_out, w_out)."""
    layers = []
    c = c_in
    width = 32
    for i in range(10):
        stride = 1 if i % 2 == 0 else 2
        if i == 0:
            c_out = width
        elif stride == 2:
            width = min(512, width * 2)
            c_out = width
        else:
            c_out = width
        ho = (h + 2 - 3) // stride + 1
        wo = (w + 2 - 3) // stride + 1
        layers.append(dict(c_in=c, c_out=c_out, stride=stride, h_in=h, w_in=w, h_out=ho, w_out=wo))
        c, h, w = c_out, ho, wo
    return layers


def cnn_weights(seed, layers, sigma=0.02):
    """Per-layer weights in K,R,S,C order (c_out,3,3,c_in), N(0, sigma^2) rounded to bf16 bits."""
    out = []
    for li, L in enumerate(layers):
        cnt = L["c_out"] * 9 * L["c_in"]
        wt = normal(seed ^ (0x1000 + li), cnt, sigma=sigma).reshape(L["c_out"], 3, 3, L["c_in"])
        out.append(f32_to_bf16_bits(wt))
    return out


def cnn_input(seed, batch, h=416, w=416, c=3):
    """NHWC input U[0,1) rounded to bf16 bits."""
    x = uniform01(seed ^ 0x77, batch * h * w * c).reshape(batch, h, w, c)
    return f32_to_bf16_bits(x)


def task_data(spec):
    """All host inputs of one task of a mix, keyed as the harness expects them."""
    k, p, seed = spec.kind, spec.params, spec.seed
    if k == "jacobi":
        return dict(u=jacobi_field(seed, p["n"]))
    if k == "gemm_f32":
        a, b = gemm_operands_f32(seed, p["m"], p["n"], p["k"])
        return dict(a=a, b=b)
    if k == "gemm_bf16":
        a, b = gemm_operands_bf16(seed, p["m"], p["n"], p["k"])
        return dict(a=a, b=b)
    if k == "bfs":
        rp, ci = er_graph_csr(seed, p["n"], p["degree"])
        return dict(row_ptr=rp, col_idx=ci)
    if k == "cnn":
        layers = cnn_layers(p["h"], p["w"])
        return dict(layers=layers, weights=cnn_weights(seed, layers), x=cnn_input(seed, p["batch"], p["h"], p["w"]))
    raise ValueError(k)
