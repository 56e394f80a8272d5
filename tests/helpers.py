"""Shared test helpers: library trace -> checker inputs, decision comparison, error metrics."""
import numpy as np

import oracle
import paper_2107_08538_amd as mgb

_KIND = {mgb.MGB_EV_ADMIT: oracle.D_ADMIT, mgb.MGB_EV_QUEUED: oracle.D_WAIT,
         mgb.MGB_EV_REJECT: oracle.D_REJECT, mgb.MGB_EV_RELEASE: oracle.D_RELEASE,
         mgb.MGB_EV_CANCELLED: oracle.D_CANCELLED, mgb.MGB_EV_GROWN: oracle.D_GROWN}
_IN = {mgb.MGB_EV_PROBE: oracle.IN_PROBE, mgb.MGB_EV_COMPLETE: oracle.IN_COMPLETE,
       mgb.MGB_EV_CANCEL: oracle.IN_CANCEL, mgb.MGB_EV_GROW: oracle.IN_GROW}


def oracle_device(desc):
    return oracle.device(desc.mem_cap_bytes, n_cu=desc.n_cu, granule_cus=desc.granule_cus,
                         wave_size=desc.wave_size, max_waves_per_cu=desc.max_waves_per_cu,
                         max_wg_per_cu=desc.max_wg_per_cu, policy=desc.policy,
                         queue_mode=desc.queue_mode, max_running=desc.max_running)


def split_trace(trace):
    """Returns (inputs for the replay, list of the library's decision records with the index of
    the input that caused each)."""
    is_in = np.isin(trace["kind"], list(_IN))
    tin = trace[is_in]
    inputs = np.zeros(len(tin), dtype=oracle.INPUT_DT)
    seq_to_index = {}
    for i, r in enumerate(tin):
        inputs[i]["kind"] = _IN[int(r["kind"])]
        inputs[i]["id"] = r["task_id"] if r["kind"] == mgb.MGB_EV_PROBE else r["ticket"]
        inputs[i]["mem"] = r["mem_bytes"]
        inputs[i]["grid"] = r["grid"]
        inputs[i]["block"] = r["block"]
        inputs[i]["wg_per_cu"] = r["demand"] if r["kind"] == mgb.MGB_EV_PROBE else 0    # the probe's residency fact
        seq_to_index[int(r["seq"])] = i
    return inputs, trace[~is_in], seq_to_index


def assert_trace_matches_replay(desc, trace):
    """Bit-exact comparison of every decision the library logged with the independent replay."""
    inputs, dec_lib, seq_to_index = split_trace(trace)
    dec = oracle.sched_replay(oracle_device(desc), inputs)
    assert len(dec) == len(dec_lib), (len(dec), len(dec_lib))
    assert np.all(np.diff(trace["seq"].astype(np.int64)) == 1) and trace["seq"][0] == 0
    assert np.all(np.diff(trace["t_ns"].astype(np.int64)) >= 0)
    for a, b in zip(dec_lib, dec):
        assert _KIND[int(a["kind"])] == b["kind"], (a, b)
        assert seq_to_index[int(a["cause_seq"])] == b["in_index"], (a, b)
        assert a["code"] == b["code"], (a, b)
        if b["kind"] == oracle.D_REJECT and b["ticket"] == 0:
            continue
        assert a["ticket"] == b["ticket"] and a["task_id"] == b["task_id"], (a, b)
        assert a["granule_mask"] == b["granule_mask"], (a, b)
        assert a["free_bytes"] == b["free_bytes"] and a["free_granules"] == b["free_granules"], (a, b)
        assert a["demand"] == b["demand"], (a, b)
        assert np.array_equal(a["cu_mask"], b["cu_mask"]), (a, b)
    return dec


def gemm_componentwise_error(c_gpu, ref, den):
    """max_ij |c - ref| / (|A||B|)_ij -- the componentwise rounding-error measure."""
    return float((np.abs(c_gpu.astype(np.float64) - ref) / den).max())


def frobenius_rel(x, ref):
    x = np.asarray(x, dtype=np.float64)
    return float(np.linalg.norm((x - ref).ravel()) / np.linalg.norm(ref.ravel()))


def verify_task_output(task, data, full_gemm_limit=512):
    """Compare one finished harness task with the CPU checker (tolerances as in the kernel tests)."""
    import workloads as W
    spec, p = task.spec, task.spec.params
    if spec.kind == "jacobi":
        it = p["iters"]
        got = (task.tensors["u0"] if it % 2 == 0 else task.tensors["u1"]).cpu().numpy()
        assert np.array_equal(got, oracle.jacobi_f32(data["u"], it)), ("jacobi", spec.task_id)
    elif spec.kind in ("gemm_f32", "gemm_bf16"):
        got = task.tensors["C"].cpu().numpy().astype(np.float64)
        m, n = got.shape
        if spec.kind == "gemm_f32":
            if max(m, n, p["k"]) <= full_gemm_limit:
                ref, den = oracle.gemm_f32(data["a"], data["b"]), oracle.gemm_abs_f32(data["a"], data["b"])
                assert (np.abs(got - ref) / den).max() <= 1e-4, ("gemm_f32", spec.task_id)
            else:
                rng = np.random.default_rng(spec.task_id)
                rows = rng.integers(0, m, 1024).astype(np.uint32)
                cols = rng.integers(0, n, 1024).astype(np.uint32)
                ref, den = oracle.gemm_f32_entries(data["a"], data["b"], rows, cols)
                assert (np.abs(got[rows, cols] - ref) / den).max() <= 1e-4, ("gemm_f32", spec.task_id)
        else:
            if max(m, n, p["k"]) <= full_gemm_limit:
                assert frobenius_rel(got, oracle.gemm_bf16(data["a"], data["b"])) <= 1e-2, ("gemm_bf16", spec.task_id)
            else:
                rng = np.random.default_rng(spec.task_id)
                rows = rng.integers(0, m, 1024).astype(np.uint32)
                cols = rng.integers(0, n, 1024).astype(np.uint32)
                ref = oracle.gemm_bf16_entries(data["a"], data["b"], rows, cols)
                assert np.linalg.norm(got[rows, cols] - ref) <= 1e-2 * np.linalg.norm(ref), ("gemm_bf16", spec.task_id)
    elif spec.kind == "bfs":
        got = task.tensors["level"].cpu().numpy()
        assert np.array_equal(got, oracle.bfs(data["row_ptr"], data["col_idx"], 0)), ("bfs", spec.task_id)
    elif spec.kind == "cnn":
        L = data["layers"]
        got = task.tensors["out"].cpu().numpy().reshape(p["batch"], L[-1]["h_out"], L[-1]["w_out"], L[-1]["c_out"])
        ref = oracle.cnn_forward(data["x"], data["weights"], [l["stride"] for l in L])
        assert frobenius_rel(got, ref) <= 1e-2, ("cnn", spec.task_id)
    else:
        raise ValueError(spec.kind)


def check_ledger_invariants(desc, trace):
    """Resident footprints never exceed the cap; HARD partitions stay pairwise disjoint."""
    running = {}
    for r in trace:
        k = int(r["kind"])
        if k == mgb.MGB_EV_ADMIT:
            for g in running.values():
                if desc.policy != mgb.MGB_POLICY_SOFT:
                    assert g[1] & int(r["granule_mask"]) == 0
            running[int(r["ticket"])] = (int(r["mem_bytes"]), int(r["granule_mask"]))
        elif k == mgb.MGB_EV_RELEASE:
            del running[int(r["ticket"])]
        assert sum(m for m, _ in running.values()) + int(r["free_bytes"]) == desc.mem_cap_bytes
    assert not running


# ------------------------------------------------------------------ checks for sizes the serial checker cannot recompute whole
def _matvec64(m, x, chunk=512):
    """m @ x in float64, converting a block of rows at a time."""
    out = np.empty(m.shape[0], dtype=np.float64)
    for i in range(0, m.shape[0], chunk):
        out[i:i + chunk] = m[i:i + chunk].astype(np.float64) @ x
    return out


def _abs_matvec64(m, x, chunk=512):
    out = np.empty(m.shape[0], dtype=np.float64)
    for i in range(0, m.shape[0], chunk):
        out[i:i + chunk] = np.abs(m[i:i + chunk].astype(np.float64)) @ x
    return out


# Freivalds' check of C = A B with one random sign vector x: C x against A (B x), both in double.
# Bound on what a correct fp32-accumulating kernel may leave: an entry of C is off by at most about
# sqrt(k) 2^-24 (|A||B|)_ij in the typical case (2.4e-4 (|A||B|)_ij at worst, never seen); the signed
# sum over a row of n such errors is smaller still relative to (|A| (|B| |x|))_i.  A tile of C that
# is wrong (not computed, computed from the wrong slab, transposed) moves (C x)_i by about
# sqrt(tile) sqrt(k) against n k 0.64, i.e. 1e-4 at 4096^3 and 4e-6 for a 256-wide tile at 32768^3;
# a single entry off by its own size moves it by 2.6e-7 even there.  Measured on the kernels:
# 3e-9 at most over the 40 products of the 128-task mix, 7e-10 at 32768^3.
FREIVALDS_TOL = 1e-7


def freivalds_ratio(a, b, c, seed):
    """max_i |(C x)_i - (A (B x))_i| / (|A| (|B| |x|))_i for a random +-1 vector x."""
    n = b.shape[1]
    x = np.random.default_rng(seed).choice(np.array([-1.0, 1.0]), size=n)
    ref = _matvec64(a, _matvec64(b, x))
    den = _abs_matvec64(a, _abs_matvec64(b, np.ones(n)))
    return float((np.abs(_matvec64(c, x) - ref) / den).max())


def band_samples(m, n, band, seed):
    """One row per band of `band` rows and one column per band of columns, at random places inside
    the bands: their products (all pairs) put at least one sample in every band x band block."""
    rng = np.random.default_rng(seed)
    rows = np.array([min(m - 1, r0 + int(rng.integers(0, band))) for r0 in range(0, m, band)], dtype=np.int64)
    cols = np.array([min(n - 1, c0 + int(rng.integers(0, band))) for c0 in range(0, n, band)], dtype=np.int64)
    return rows, cols


def bf16_bits_to_f32(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32)


def jacobi_cone_points(n, iters, seed, extra=3):
    rng = np.random.default_rng(seed)
    pts = [(1, 1), (n - 2, n - 2), (1, n // 2), (n // 2, n - 2)]
    pts += [(int(rng.integers(1, n - 1)), int(rng.integers(1, n - 1))) for _ in range(extra)]
    return pts


def jacobi_cone_check(u_init, result_at, n, iters, points):
    """A cell after `iters` sweeps depends on the initial cells within distance `iters`: recompute
    each sampled cell from that window of the initial grid (square, shifted not clipped at the rim,
    so that a fixed rim of the window is either the grid's own ring or out of reach) and compare
    bit for bit.  u_init(r0, r1, c0, c1) returns the window, result_at(r, c) the kernel's value."""
    side = min(n, 2 * iters + 3)
    for (r, c) in points:
        r0 = min(max(0, r - iters - 1), n - side)
        c0 = min(max(0, c - iters - 1), n - side)
        patch = np.ascontiguousarray(u_init(r0, r0 + side, c0, c0 + side))
        want = oracle.jacobi_f32(patch, iters)[r - r0, c - c0]
        assert float(result_at(r, c)) == float(want), ("jacobi", n, r, c)


def verify_task_output_at_full_size(task, data, seed=0):
    """Every kind at sizes the serial checker cannot recompute whole: Jacobi on dependency cones of
    sampled cells (bit-exact), GEMM on a sample in every 64 x 64 block of C plus Freivalds' check
    of the whole product, BFS in full (bit-exact).  Returns the Freivalds ratio of a GEMM, else None."""
    spec, p = task.spec, task.spec.params
    if spec.kind == "jacobi":
        n, it = p["n"], p["iters"]
        res = task.tensors["u0"] if it % 2 == 0 else task.tensors["u1"]
        pts = jacobi_cone_points(n, it, seed + spec.task_id)
        vals = res[[r for r, _ in pts], [c for _, c in pts]].cpu().numpy()
        look = {pt: v for pt, v in zip(pts, vals)}
        u = data["u"]
        jacobi_cone_check(lambda r0, r1, c0, c1: u[r0:r1, c0:c1], lambda r, c: look[(r, c)], n, it, pts)
        ring = torch_ring_max(res)
        assert ring == 0.0, ("jacobi ring", spec.task_id)
        return None
    if spec.kind in ("gemm_f32", "gemm_bf16"):
        m, n = p["m"], p["n"]
        c = task.tensors["C"].cpu().numpy()
        rows, cols = band_samples(m, n, 64, seed + spec.task_id)
        rr, cc = np.meshgrid(rows, cols, indexing="ij")
        rr, cc = rr.ravel().astype(np.uint32), cc.ravel().astype(np.uint32)
        got = c[rr, cc].astype(np.float64)
        if spec.kind == "gemm_f32":
            ref, den = oracle.gemm_f32_entries(data["a"], data["b"], rr, cc)
            assert (np.abs(got - ref) / den).max() <= 1e-4, ("gemm_f32", spec.task_id)
            a, b = data["a"], data["b"]
        else:
            ref = oracle.gemm_bf16_entries(data["a"], data["b"], rr, cc)
            assert np.linalg.norm(got - ref) <= 1e-2 * np.linalg.norm(ref), ("gemm_bf16", spec.task_id)
            a, b = bf16_bits_to_f32(data["a"]), bf16_bits_to_f32(data["b"])
        ratio = freivalds_ratio(a, b, c, seed + spec.task_id)
        assert ratio <= FREIVALDS_TOL, (spec.kind, spec.task_id, ratio)
        return ratio
    if spec.kind == "bfs":
        got = task.tensors["level"].cpu().numpy()
        assert np.array_equal(got, oracle.bfs(data["row_ptr"], data["col_idx"], 0)), ("bfs", spec.task_id)
        return None
    raise ValueError(spec.kind)


def torch_ring_max(t):
    import torch
    return float(torch.stack([t[0, :].abs().max(), t[-1, :].abs().max(), t[:, 0].abs().max(), t[:, -1].abs().max()]).max())


# ------------------------------------------------------------------ the conv net at 416 x 416: output pixels through their receptive field
def cnn_patch_for(oy, ox, h_in, w_in, total_stride=32, reach=2):
    """Rows / columns of the input image that decide output pixel (oy, ox) of the 10-layer net, as a
    window aligned to the net's total stride: going back through the layers, output row i of a
    stride-2 layer reads rows 2i-1 .. 2i+1 and of a stride-1 layer i-1 .. i+1, so row i of the last
    layer reads input rows 32 i - 62 .. 32 i + 62.  The window [32 (i - 2), 32 (i + 2)) holds them;
    clipped at the image it ends where the image ends, so that the window's zero padding is the
    image's own padding there, and it starts at a multiple of 32, so that every layer's stride
    pattern falls on the same pixels as in the whole image."""
    y0, y1 = max(0, total_stride * (oy - reach)), min(h_in, total_stride * (oy + reach))
    x0, x1 = max(0, total_stride * (ox - reach)), min(w_in, total_stride * (ox + reach))
    return y0, y1, x0, x1, oy - y0 // total_stride, ox - x0 // total_stride
