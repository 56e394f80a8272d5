"""Shared test helpers: library trace -> checker inputs, decision comparison, error metrics."""
import numpy as np

import oracle
import paper_2107_08538_amd as mgb

_KIND = {mgb.MGB_EV_ADMIT: oracle.D_ADMIT, mgb.MGB_EV_QUEUED: oracle.D_WAIT,
         mgb.MGB_EV_REJECT: oracle.D_REJECT, mgb.MGB_EV_RELEASE: oracle.D_RELEASE,
         mgb.MGB_EV_CANCELLED: oracle.D_CANCELLED}
_IN = {mgb.MGB_EV_PROBE: oracle.IN_PROBE, mgb.MGB_EV_COMPLETE: oracle.IN_COMPLETE,
       mgb.MGB_EV_CANCEL: oracle.IN_CANCEL}


def oracle_device(desc):
    return oracle.device(desc.mem_cap_bytes, n_cu=desc.n_cu, granule_cus=desc.granule_cus,
                         wave_size=desc.wave_size, max_waves_per_cu=desc.max_waves_per_cu,
                         max_wg_per_cu=desc.max_wg_per_cu, policy=desc.policy,
                         queue_mode=desc.queue_mode)


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
