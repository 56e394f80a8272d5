"""Multi-process front end (Sec. IV) without a GPU: clients in threads and in separate processes
reach one scheduler over shared memory; every decision replays; a dead client's tasks come back."""
import os
import subprocess
import sys
import threading
import time

import numpy as np
import pytest

import oracle
import paper_2107_08538_amd as mgb
from helpers import assert_trace_matches_replay

HERE = os.path.dirname(os.path.abspath(__file__))
CHILD = os.path.join(HERE, "ipc_children.py")


def _name(tag):
    return "t%d_%s" % (os.getpid(), tag)


def _sched(**kw):
    kw.setdefault("granule_cus", 8)
    return mgb.Sched(backend=mgb.MGB_BACKEND_NULL, **kw)


def test_protocol_in_one_process():
    s = _sched(mem_cap_bytes=1000)
    name = _name("proto")
    sv = mgb.Server(s, name, 2)
    with pytest.raises(mgb.MgbError):
        mgb.Server(s, name, 2)                               # the name is taken
    with pytest.raises(mgb.MgbError):
        mgb.Client(_name("nobody"))
    c1, c2 = mgb.Client(name), mgb.Client(name)
    with pytest.raises(mgb.MgbError):
        mgb.Client(name)                                     # both slots are taken
    rc, p1 = c1.probe(1, 700, (128, 1, 1), (256, 1, 1), wg_per_cu=2)          # 8 per CU by wave slots, 2 by its own resources
    assert rc == mgb.MGB_OK and p1.n_granules == 8 and p1.granule_mask == 0xFF and p1.cu_mask[0] == 0xFFFFFFFF
    assert p1.stream is None
    rc, p2 = c2.probe(2, 700, (8, 1, 1), (64, 1, 1))
    assert rc == mgb.MGB_WAIT
    assert c2.wait(p2.ticket, 1_000_000)[0] == mgb.MGB_TIMEOUT
    assert c1.grow(p1.ticket, 300) == mgb.MGB_OK and c1.grow(p1.ticket, 1) == mgb.MGB_E_BUSY
    assert c2.stats().free_bytes == 0 and c2.stats().n_waiting == 1
    assert c1.disconnect() == mgb.MGB_E_BUSY                 # still holds a task
    got = []
    th = threading.Thread(target=lambda: got.append(c2.wait(p2.ticket)))
    th.start()
    time.sleep(0.05)
    assert c1.complete(p1.ticket) == mgb.MGB_OK
    th.join(10)
    assert got and got[0][0] == mgb.MGB_OK and got[0][1].ticket == p2.ticket
    assert c2.complete(p2.ticket) == mgb.MGB_OK and c2.complete(p2.ticket) == mgb.MGB_E_UNKNOWN_TICKET
    assert c1.disconnect() == mgb.MGB_OK and c2.disconnect() == mgb.MGB_OK
    c3 = mgb.Client(name)                                    # a freed slot can be claimed again
    assert c3.disconnect() == mgb.MGB_OK
    assert sv.stop() == mgb.MGB_OK
    assert_trace_matches_replay(s.desc, s.trace())
    assert s.stats().free_bytes == 1000 and s.destroy() == mgb.MGB_OK


def test_independent_processes_share_one_scheduler():
    s = _sched(mem_cap_bytes=1500)
    name = _name("procs")
    sv = mgb.Server(s, name, 8)
    procs = [subprocess.Popen([sys.executable, CHILD, "storm", name, str(seed), "40"]) for seed in (1, 2, 3, 4)]
    for p in procs:
        assert p.wait(timeout=120) == 0
    assert sv.reclaimed() == 0
    assert sv.stop() == mgb.MGB_OK
    tr = s.trace()
    dec = assert_trace_matches_replay(s.desc, tr)
    assert (dec["kind"] == oracle.D_ADMIT).sum() == 160 and (dec["kind"] == oracle.D_RELEASE).sum() == 160
    assert s.stats().free_bytes == 1500 and s.stats().n_running == 0
    assert s.destroy() == mgb.MGB_OK


def test_a_dead_client_gives_everything_back():
    s = _sched(mem_cap_bytes=1000)
    name = _name("dead")
    sv = mgb.Server(s, name, 4)
    p = subprocess.Popen([sys.executable, CHILD, "hold_and_die", name, "600"], stdout=subprocess.PIPE, text=True)
    assert p.stdout.readline().strip() == "holding"
    c = mgb.Client(name)
    st = c.stats()
    assert (st.free_bytes, st.n_running, st.n_waiting) == (400, 1, 1)
    rc, pl = c.probe(1, 900, (8, 1, 1), (64, 1, 1))          # waits behind what the other process holds
    assert rc == mgb.MGB_WAIT
    assert p.wait(timeout=30) == 0
    rc, pl = c.wait(pl.ticket, 5_000_000_000)                # admitted once the server has noticed the death
    assert rc == mgb.MGB_OK
    assert sv.reclaimed() == 2                               # one resident task completed, one queued probe withdrawn
    assert c.complete(pl.ticket) == mgb.MGB_OK and c.disconnect() == mgb.MGB_OK
    assert sv.stop() == mgb.MGB_OK
    assert s.stats().free_bytes == 1000 and s.stats().n_running == 0 and s.stats().n_waiting == 0
    assert_trace_matches_replay(s.desc, s.trace())
    assert s.destroy() == mgb.MGB_OK


def test_clients_notice_a_server_that_stopped():
    s = _sched(mem_cap_bytes=1000)
    name = _name("stop")
    sv = mgb.Server(s, name, 2)
    c = mgb.Client(name)
    assert sv.stop() == mgb.MGB_OK
    rc, pl = c.probe(1, 10, (1, 1, 1), (64, 1, 1))
    assert rc == mgb.MGB_E_BACKEND
    assert s.destroy() == mgb.MGB_OK


def test_two_threads_share_one_connection_while_one_waits():
    # the waiter must not keep the connection to itself: the completion that lets it in comes
    # from another thread of the same process, over the same connection
    s = _sched(mem_cap_bytes=1000)
    name = _name("share")
    sv = mgb.Server(s, name, 1)
    c = mgb.Client(name)
    rc, p1 = c.probe(1, 700, (8, 1, 1), (64, 1, 1))
    assert rc == mgb.MGB_OK
    rc, p2 = c.probe(2, 700, (8, 1, 1), (64, 1, 1))
    assert rc == mgb.MGB_WAIT
    got = []
    th = threading.Thread(target=lambda: got.append(c.wait(p2.ticket, 20_000_000_000)))
    th.start()
    time.sleep(0.1)                                          # the waiter is inside its wait
    assert c.stats().n_waiting == 1
    assert c.complete(p1.ticket) == mgb.MGB_OK
    th.join(30)
    assert not th.is_alive() and got[0][0] == mgb.MGB_OK and got[0][1].ticket == p2.ticket
    assert c.complete(p2.ticket) == mgb.MGB_OK
    assert c.disconnect() == mgb.MGB_OK
    sv.stop()
    assert_trace_matches_replay(s.desc, s.trace())
    assert s.destroy() == 0


@pytest.mark.parametrize("granule_cus", [1, 2, 4])
def test_client_refuses_to_build_a_stream_for_a_mask_that_misses_an_xcd(granule_cus):
    # mask bit i is a CU of XCD (i mod 8): a server that only decides may hand out granules of fewer
    # than 8 CUs, and such a mask must be refused before the runtime sees it (no GPU call is reached)
    s = mgb.Sched(backend=mgb.MGB_BACKEND_NULL, n_cu=32 * granule_cus, granule_cus=granule_cus)
    name = _name("xcd%d" % granule_cus)
    sv = mgb.Server(s, name, 1)
    c = mgb.Client(name)
    rc, pl = c.probe(1, 10, (1, 1, 1), (64, 1, 1))
    assert rc == mgb.MGB_OK and pl.granule_mask == 1 and pl.cu_mask[0] == (1 << granule_cus) - 1
    rc, st = c.stream(pl)
    assert rc == mgb.MGB_E_INVAL and not st.value
    assert b"XCD" in mgb.mgb_last_error()
    # seven of the eight residues are not enough either; an empty mask was refused before
    pl.cu_mask[0] = 0x7F7F7F7F
    assert c.stream(pl)[0] == mgb.MGB_E_INVAL
    for k in range(8):
        pl.cu_mask[k] = 0
    assert c.stream(pl)[0] == mgb.MGB_E_INVAL
    assert c.complete(pl.ticket) == mgb.MGB_OK and c.disconnect() == mgb.MGB_OK
    assert sv.stop() == mgb.MGB_OK and s.destroy() == mgb.MGB_OK


def test_a_slot_is_free_only_after_its_owner_collected_the_goodbye():
    # connect / disconnect in a tight loop from several threads on fewer slots than threads: a client
    # that claimed a slot whose previous owner had not yet read its answer would see a stale status
    s = _sched()
    name = _name("bye")
    sv = mgb.Server(s, name, 2)
    bad = []

    def churn(k):
        for i in range(150):
            try:
                c = mgb.Client(name)
            except mgb.MgbError:
                continue                                            # both slots taken right now
            rc, pl = c.probe(k * 1000 + i, 1, (1, 1, 1), (64, 1, 1))
            if rc != mgb.MGB_OK or pl.ticket == 0:
                bad.append(("probe", rc))
            elif c.complete(pl.ticket) != mgb.MGB_OK:
                bad.append(("complete", k, i))
            if c.disconnect() != mgb.MGB_OK:
                bad.append(("bye", k, i))
    th = [threading.Thread(target=churn, args=(k,)) for k in range(4)]
    [t.start() for t in th]
    [t.join() for t in th]
    assert not bad, bad[:5]
    assert sv.stop() == mgb.MGB_OK and s.destroy() == mgb.MGB_OK
