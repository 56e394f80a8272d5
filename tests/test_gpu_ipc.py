"""Multi-process front end on the GPU: independent processes, each with its own HIP context, get
placements from one scheduler process and run on their own CU-masked streams."""
import os
import subprocess
import sys

import pytest

import oracle
from helpers import assert_trace_matches_replay

pytestmark = pytest.mark.gpu

import paper_2107_08538_amd as mgb  # noqa: E402

CHILD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "ipc_children.py")


def test_three_processes_run_tasks_under_masks_from_one_scheduler():
    # the scheduler process only decides (null backend: it never touches the device)
    s = mgb.Sched(backend=mgb.MGB_BACKEND_NULL)
    name = "g%d" % os.getpid()
    sv = mgb.Server(s, name, 4)
    kinds = ("jacobi", "gemm", "jacobi")
    procs = [subprocess.Popen([sys.executable, CHILD, "gpu_task", name, k, str(10 + i)], stdout=subprocess.PIPE,
                              stderr=subprocess.PIPE, text=True) for i, k in enumerate(kinds)]
    outs = [p.communicate(timeout=280) for p in procs]
    for p, (so, se), k in zip(procs, outs, kinds):
        assert p.returncode == 0, (k, so[-500:], se[-1500:])
        assert so.strip().startswith("ok " + k)
    assert sv.reclaimed() == 0 and sv.stop() == mgb.MGB_OK
    dec = assert_trace_matches_replay(s.desc, s.trace())
    assert (dec["kind"] == oracle.D_ADMIT).sum() == 3 and (dec["kind"] == oracle.D_RELEASE).sum() == 3
    assert s.stats().free_bytes == s.desc.mem_cap_bytes
    assert s.destroy() == mgb.MGB_OK
