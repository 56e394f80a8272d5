"""Whole task mixes through the scheduler on the GPU: every output against the CPU checker, every
decision against the replay.  Mix-16 runs at its full size; CNN-8 and Mixed-128 run on reduced
instances that the serial checker can recompute in seconds."""
import numpy as np
import pytest

import oracle
import workloads as W
from helpers import assert_trace_matches_replay, check_ledger_invariants, verify_task_output

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

import paper_2107_08538_amd as mgb  # noqa: E402
from paper_2107_08538_amd import harness  # noqa: E402


def _run(spec, use_arrivals=True, time_scale=1.0, **sched_kw):
    data = [W.task_data(t) for t in spec["tasks"]]
    tasks = [harness.build_task(t, d) for t, d in zip(spec["tasks"], data)]
    cap = min(spec["cap_bytes"], torch.cuda.mem_get_info()[1])
    s = mgb.Sched(mem_cap_bytes=cap, **sched_kw)
    rec, makespan = harness.run_mix(s, tasks, use_arrivals=use_arrivals, time_scale=time_scale)
    return s, tasks, data, rec


def test_mix16_full_size_outputs_and_decisions():
    s, tasks, data, rec = _run(W.mix16())
    assert sorted(t.spec.kind for t in tasks).count("jacobi") >= 1
    for t, d in zip(tasks, data):
        verify_task_output(t, d)
    trace = s.trace()
    dec = assert_trace_matches_replay(s.desc, trace)
    check_ledger_invariants(s.desc, trace)
    assert (dec["kind"] == oracle.D_ADMIT).sum() == 16
    # demand the probes carried: GEMM 4096^3 and Jacobi 4096^2 = the whole device, BFS 2^20 = half
    want = {"gemm_f32": 32, "jacobi": 32, "bfs": 16}
    for r, t in zip(rec, tasks):
        assert r["granules"] == want[t.spec.kind]
    assert s.destroy() == 0


@pytest.mark.parametrize("policy", [mgb.MGB_POLICY_HARD, mgb.MGB_POLICY_SOFT, mgb.MGB_POLICY_SERIAL])
def test_mix16_batch_at_t0_all_policies(policy):
    # all 16 probes issued before anything runs (the paper's batch setting): queues must form
    s, tasks, data, rec = _run(W.mix16(seed=3), use_arrivals=False, policy=policy)
    for t, d in zip(tasks, data):
        if t.spec.kind != "jacobi":             # Jacobi is covered at full size above
            verify_task_output(t, d)
    trace = s.trace()
    dec = assert_trace_matches_replay(s.desc, trace)
    check_ledger_invariants(s.desc, trace)
    waits = (dec["kind"] == oracle.D_WAIT).sum()
    if policy == mgb.MGB_POLICY_SERIAL:
        assert waits == 15
    elif policy == mgb.MGB_POLICY_HARD:
        assert waits > 0
    else:
        assert waits == 0                       # memory never binds here and compute is soft
    assert s.destroy() == 0


def test_cnn8_reduced_images():
    s, tasks, data, rec = _run(W.cnn8(h=52, w=52), time_scale=0.1)
    assert {t.spec.params["batch"] for t in tasks} <= {1, 2, 4, 8}
    for t, d in zip(tasks, data):
        verify_task_output(t, d)
    trace = s.trace()
    assert_trace_matches_replay(s.desc, trace)
    check_ledger_invariants(s.desc, trace)
    assert s.destroy() == 0


def test_mixed128_reduced_sizes():
    spec = W.mixed128(shrink=16)
    kinds = {t.kind for t in spec["tasks"]}
    assert kinds == {"jacobi", "gemm_f32", "gemm_bf16", "bfs"} and len(spec["tasks"]) == 128
    s, tasks, data, rec = _run(spec, time_scale=0.25)
    for t, d in zip(tasks, data):
        verify_task_output(t, d)
    trace = s.trace()
    dec = assert_trace_matches_replay(s.desc, trace)
    check_ledger_invariants(s.desc, trace)
    assert (dec["kind"] == oracle.D_ADMIT).sum() == 128
    grids = sorted(int(r["grid"][0]) for r in trace if r["kind"] == mgb.MGB_EV_PROBE)
    assert grids[0] == 8 and grids[-1] > grids[0]     # a range of small grids that share the device
    assert s.destroy() == 0
