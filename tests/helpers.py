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
