"""Pins for the CPU checker's scheduler replay: a hand-worked trace, invariants
that hold after every event, degenerate policies, and a literal thread-block
by thread-block emulation of Algorithm 2's residency test for the demand rule."""
import itertools
import json
import os

import numpy as np
import pytest

import oracle
from oracle import (D_ADMIT, D_WAIT, D_REJECT, D_RELEASE, D_CANCELLED, D_GROWN, POL_HARD, POL_SOFT,
                    POL_SERIAL, POL_CG, Q_BACKFILL, Q_FIFO)

GOLD = os.path.join(os.path.dirname(__file__), "golden", "sched_hand_case.json")
KIND = {"admit": D_ADMIT, "wait": D_WAIT, "reject": D_REJECT, "release": D_RELEASE}


def _events(raw):
    out = []
    for ev in raw:
        if ev[0] == "probe":
            out.append(("probe", ev[1], ev[2], tuple(ev[3]), tuple(ev[4])))
        else:
            out.append((ev[0], ev[1]))
    return out


@pytest.mark.parametrize("mode,key", [(Q_BACKFILL, "backfill"), (Q_FIFO, "fifo")])
def test_hand_worked_trace(mode, key):
    g = json.load(open(GOLD))
    dev = oracle.device(policy=POL_HARD, queue_mode=mode, **g["device"])
    dec = oracle.sched_replay(dev, oracle.make_inputs(_events(g["events"])))
    want = g[key]
    assert len(dec) == len(want)
    for d, w in zip(dec, want):
        assert d["in_index"] == w["in"] and d["kind"] == KIND[w["kind"]], (d, w)
        if w["kind"] == "reject":
            assert d["code"] == w["code"]
            continue
        assert d["ticket"] == w["ticket"] and d["task_id"] == w["task_id"]
        assert d["demand"] == w["demand"] and d["granule_mask"] == w["granules"]
        assert d["cu_mask"][0] == w["cu_mask0"] and not d["cu_mask"][1:].any()
        assert d["free_bytes"] == w["free_bytes"] and d["free_granules"] == w["free_granules"]


# ---- the demand rule against a literal emulation of Algorithm 2 -----------------------------
def _alg2_places_all(n_sm, blocks, warps_per_block, max_tb, max_warps):
    """Place thread blocks one at a time, round-robin over SMs, honouring the per-SM limits on
    resident blocks and warps; succeed iff every block found a slot (empty device)."""
    tb = [0] * n_sm
    wp = [0] * n_sm
    nxt = 0
    for _ in range(blocks):
        placed = False
        for probe in range(n_sm):
            s = (nxt + probe) % n_sm
            if tb[s] < max_tb and wp[s] + warps_per_block <= max_warps:
                tb[s] += 1
                wp[s] += warps_per_block
                nxt = (s + 1) % n_sm
                placed = True
                break
        if not placed:
            return False
    return True


@pytest.mark.parametrize("threads", [1, 64, 65, 128, 256, 448, 512, 1024])
@pytest.mark.parametrize("max_tb,max_warps", [(32, 32), (8, 32), (16, 40), (2, 10)])
def test_demand_is_smallest_device_that_holds_all_blocks(threads, max_tb, max_warps):
    n_cu = 24
    dev = oracle.device(1 << 30, n_cu=n_cu, granule_cus=1, max_waves_per_cu=max_warps,
                        max_wg_per_cu=max_tb)
    wpb = -(-threads // 64)
    for blocks in [1, 2, 7, 8, 9, 31, 32, 33, 64, 100, 191, 192, 193, 500]:
        d, waves = oracle.demand(dev, (blocks, 1, 1), (threads, 1, 1))
        assert waves == blocks * wpb
        if wpb > max_warps:
            # a block larger than a CU's wave budget: the rule still grants one block per CU
            assert d == min(n_cu, blocks)
            continue
        fits = [c for c in range(1, n_cu + 1) if _alg2_places_all(c, blocks, wpb, max_tb, max_warps)]
        want = fits[0] if fits else n_cu        # never fits => whole device (clamped)
        assert d == want, (threads, blocks, d, want)


@pytest.mark.parametrize("hint", [1, 2, 3, 5, 40])
def test_demand_with_the_tasks_own_residency_limit(hint):
    # a task whose registers / LDS allow `hint` workgroups per CU: the thread-block-by-thread-block
    # emulation with that limit on resident blocks, against the rule
    n_cu, max_tb, max_warps = 24, 16, 32
    dev = oracle.device(1 << 30, n_cu=n_cu, granule_cus=1, max_waves_per_cu=max_warps, max_wg_per_cu=max_tb)
    for threads in (64, 256, 512):
        wpb = -(-threads // 64)
        for blocks in (1, 2, 7, 24, 25, 48, 49, 100, 383, 384, 385, 1000):
            d, _ = oracle.demand(dev, (blocks, 1, 1), (threads, 1, 1), wg_per_cu=hint)
            tb = min(max_tb, hint)
            smallest = next((c for c in range(1, n_cu + 1) if _alg2_places_all(c, blocks, wpb, tb, max_warps)), n_cu)
            assert d == smallest, (threads, blocks, d, smallest)
    # 0 = not known = the device limits alone
    assert oracle.demand(dev, (100, 1, 1), (256, 1, 1), wg_per_cu=0) == oracle.demand(dev, (100, 1, 1), (256, 1, 1))


def test_demand_uses_all_three_dimensions_and_granule_rounding():
    dev = oracle.device(1 << 30)               # 256 CUs, granules of 8, 256 threads -> 8 wg/CU
    assert oracle.demand(dev, (4, 4, 4), (16, 4, 4))[0] == 1         # 64 wg -> 8 CUs -> 1 granule
    assert oracle.demand(dev, (65, 1, 1), (256, 1, 1))[0] == 2       # 9 CUs -> 2 granules
    assert oracle.demand(dev, (1024, 1, 1), (256, 1, 1))[0] == 16
    assert oracle.demand(dev, (10 ** 6, 1, 1), (256, 1, 1))[0] == 32  # clamped to the device


# ---- invariants on random traces ------------------------------------------------------------
def _random_trace(rng, n_tasks, cap, with_cancel):
    events, live = [], []
    ticket = 0
    pending = n_tasks
    while pending or live:
        if pending and (not live or rng.random() < 0.55):
            mem = int(rng.integers(1, cap // 2))
            if rng.random() < 0.05:
                mem = cap + 1
            grid = (int(rng.integers(0 if rng.random() < 0.03 else 1, 3000)), int(rng.integers(1, 3)), 1)
            block = (int(rng.choice([64, 128, 256, 512, 1024])), 1, 1)
            events.append(("probe", 1000 + pending, mem, grid, block))
            if mem <= cap and grid[0] > 0:
                ticket += 1
                live.append(ticket)
            pending -= 1
        else:
            t = live[int(rng.integers(0, len(live)))]
            if with_cancel and rng.random() < 0.2:
                events.append(("cancel", t))
            else:
                events.append(("complete", t))
            live.remove(t)      # may be rejected (still waiting); then it stays live in the replay
    # finish everything that an early complete/cancel could not finish
    for _ in range(ticket):          # a chain of waiters may need one round each
        for t in range(1, ticket + 1):
            events.append(("complete", t))
    return events


@pytest.mark.parametrize("policy", [POL_HARD, POL_SOFT, POL_SERIAL])
@pytest.mark.parametrize("mode", [Q_BACKFILL, Q_FIFO])
@pytest.mark.parametrize("seed", range(6))
def test_invariants_after_every_event(policy, mode, seed):
    rng = np.random.default_rng(seed)
    cap = 10_000
    dev = oracle.device(cap, policy=policy, queue_mode=mode)
    events = _random_trace(rng, 40, cap, with_cancel=True)
    inputs = oracle.make_inputs(events)
    dec = oracle.sched_replay(dev, inputs)
    running = {}          # ticket -> (mem, granules)
    waiting = set()
    mem_of = {}
    for d in dec:
        k, t = d["kind"], int(d["ticket"])
        if k == D_ADMIT:
            ev = events[d["in_index"]]
            if ev[0] == "probe":
                mem_of[t] = ev[2]
            waiting.discard(t)
            running[t] = (mem_of[t], int(d["granule_mask"]))
            # buddy block: demand rounded up to a power of two, contiguous, aligned to its size
            b = 1
            while b < d["demand"]:
                b *= 2
            gm = int(d["granule_mask"])
            low = (gm & -gm).bit_length() - 1
            assert gm == ((1 << b) - 1) << low and low % b == 0
            if policy == POL_SERIAL:
                assert d["granule_mask"] == 0xFFFFFFFF and len(running) == 1
        elif k == D_WAIT:
            mem_of[t] = events[d["in_index"]][2]
            waiting.add(t)
        elif k == D_RELEASE:
            assert t in running
            del running[t]
        elif k == D_CANCELLED:
            assert t in waiting
            waiting.discard(t)
        # memory safety: resident footprints never exceed the cap, ledger balances
        resident = sum(m for m, _ in running.values())
        assert resident <= cap
        assert d["free_bytes"] + resident == cap
        if policy != POL_SOFT:
            masks = [g for _, g in running.values()]
            union = 0
            for g in masks:
                assert union & g == 0            # partitions pairwise disjoint
                union |= g
            assert d["free_granules"] == (~union & 0xFFFFFFFF)
        # CU mask is exactly the granules' bits
        want = np.zeros(8, dtype=np.uint32)
        for g in range(32):
            if d["granule_mask"] >> g & 1:
                want[g // 4] |= np.uint32(0xFF << (8 * (g % 4)))
        assert np.array_equal(d["cu_mask"], want)
    # liveness: the trace completes every admitted task, so nothing is left
    assert not running and not waiting
    assert dec[-1]["free_bytes"] == cap


def test_backfill_never_leaves_a_fitting_waiter_behind():
    # after any decision batch, no waiting task fits what is free (work-conserving retry)
    rng = np.random.default_rng(42)
    cap = 5000
    dev = oracle.device(cap, policy=POL_HARD, queue_mode=Q_BACKFILL)
    events = _random_trace(rng, 60, cap, with_cancel=False)
    dec = oracle.sched_replay(dev, oracle.make_inputs(events))
    waiting = {}
    last_of_input = {}
    for i, d in enumerate(dec):
        last_of_input[int(d["in_index"])] = i
    for i, d in enumerate(dec):
        t = int(d["ticket"])
        if d["kind"] == D_WAIT:
            waiting[t] = (events[d["in_index"]][2], int(d["demand"]))
        elif d["kind"] == D_ADMIT:
            waiting.pop(t, None)
        if last_of_input[int(d["in_index"])] == i:
            free_g = bin(int(d["free_granules"])).count("1")
            for mem, dem in waiting.values():
                assert mem > d["free_bytes"] or dem > free_g


# ---- degenerate policies ----------------------------------------------------------------------
def test_whole_device_demand_is_strictly_serial_in_arrival_order():
    dev = oracle.device(1 << 40, policy=POL_HARD)
    ev = [("probe", i, 10, (100000, 1, 1), (256, 1, 1)) for i in range(5)]
    ev += [("complete", t) for t in (1, 2, 3, 4, 5)]
    dec = oracle.sched_replay(dev, oracle.make_inputs(ev))
    admits = [int(d["ticket"]) for d in dec if d["kind"] == D_ADMIT]
    assert admits == [1, 2, 3, 4, 5]
    # each admission (after the first) happens at the completion of its predecessor
    assert [int(d["in_index"]) for d in dec if d["kind"] == D_ADMIT] == [0, 5, 6, 7, 8]
    # SERIAL policy gives the same schedule whatever the geometry
    dev2 = oracle.device(1 << 40, policy=POL_SERIAL)
    ev2 = [("probe", i, 10, (1, 1, 1), (64, 1, 1)) for i in range(5)] + ev[5:]
    dec2 = oracle.sched_replay(dev2, oracle.make_inputs(ev2))
    assert [(int(d["in_index"]), int(d["kind"]), int(d["ticket"])) for d in dec2] == \
           [(int(d["in_index"]), int(d["kind"]), int(d["ticket"])) for d in dec]


def test_small_tasks_unbounded_memory_all_admitted_on_arrival():
    dev = oracle.device(1 << 60, policy=POL_HARD)
    ev = [("probe", i, 1 << 30, (8, 1, 1), (256, 1, 1)) for i in range(32)]
    dec = oracle.sched_replay(dev, oracle.make_inputs(ev))
    assert all(d["kind"] == D_ADMIT for d in dec)
    assert [int(d["granule_mask"]) for d in dec] == [1 << i for i in range(32)]   # lowest free first
    # the 33rd has no granule left
    dec = oracle.sched_replay(dev, oracle.make_inputs(ev + [("probe", 99, 1, (1, 1, 1), (64, 1, 1))]))
    assert dec[-1]["kind"] == D_WAIT


def test_soft_compute_is_memory_only_admission_on_least_loaded_granules():
    dev = oracle.device(1000, policy=POL_SOFT)
    ev = [("probe", 0, 400, (100000, 1, 1), (256, 1, 1)),      # wants the whole device
          ("probe", 1, 400, (64, 1, 1), (256, 1, 1)),          # admitted anyway (compute is soft)
          ("probe", 2, 400, (64, 1, 1), (256, 1, 1)),          # memory full -> waits
          ("complete", 1), ("complete", 2), ("complete", 3)]
    dec = oracle.sched_replay(dev, oracle.make_inputs(ev))
    assert dec[0]["kind"] == D_ADMIT and dec[0]["granule_mask"] == 0xFFFFFFFF
    assert dec[1]["kind"] == D_ADMIT and dec[1]["granule_mask"] == 1      # all equally loaded -> lowest
    assert dec[2]["kind"] == D_WAIT
    # after task 0 leaves, granule 0 still carries task 1's waves: task 2 goes to granule 1
    adm = [d for d in dec if d["kind"] == D_ADMIT and d["ticket"] == 3][0]
    assert adm["in_index"] == 3 and adm["granule_mask"] == 2


def test_soft_load_is_the_tasks_waves_spread_over_its_block():
    # hand-worked: 4 CUs in granules of one, 64 wave slots each.  A (100 waves on a block of two)
    # adds ceil(100 / 2) = 50 to granules 0 and 1; B and C (60 waves, one granule each) go to the
    # empty granules 2 and 3; D then finds 50, 50, 60, 60 and takes granule 0.  Were A's 100 waves
    # charged to each of its granules, D would go to granule 2.
    dev = oracle.device(1 << 30, n_cu=4, granule_cus=1, max_waves_per_cu=64, max_wg_per_cu=64, policy=POL_SOFT)
    ev = [("probe", 0, 1, (100, 1, 1), (64, 1, 1)), ("probe", 1, 1, (60, 1, 1), (64, 1, 1)),
          ("probe", 2, 1, (60, 1, 1), (64, 1, 1)), ("probe", 3, 1, (10, 1, 1), (64, 1, 1))]
    dec = oracle.sched_replay(dev, oracle.make_inputs(ev))
    assert [d["kind"] for d in dec] == [D_ADMIT] * 4
    assert [d["demand"] for d in dec] == [2, 1, 1, 1]
    assert [d["granule_mask"] for d in dec] == [0b0011, 0b0100, 0b1000, 0b0001]


def test_fifo_release_stops_at_a_head_that_does_not_fit():
    # hand-worked: 4 granules.  A and B hold two each, C wants all four and waits, D wants one and
    # queues behind it.  When A leaves, C still does not fit: a FIFO queue admits nobody (D stays
    # behind C although two granules are free), a backfilling queue admits D at once.
    dev_kw = dict(n_cu=4, granule_cus=1, max_waves_per_cu=32, max_wg_per_cu=32, policy=POL_HARD)
    ev = [("probe", 0, 1, (64, 1, 1), (64, 1, 1)), ("probe", 1, 1, (64, 1, 1), (64, 1, 1)),
          ("probe", 2, 1, (128, 1, 1), (64, 1, 1)), ("probe", 3, 1, (1, 1, 1), (64, 1, 1)),
          ("complete", 1), ("complete", 2), ("complete", 3)]
    dec = oracle.sched_replay(oracle.device(1 << 30, queue_mode=Q_FIFO, **dev_kw), oracle.make_inputs(ev))
    got = [(int(d["in_index"]), int(d["kind"]), int(d["ticket"]), int(d["granule_mask"])) for d in dec]
    assert got == [(0, D_ADMIT, 1, 0b0011), (1, D_ADMIT, 2, 0b1100), (2, D_WAIT, 3, 0), (3, D_WAIT, 4, 0),
                   (4, D_RELEASE, 1, 0b0011),
                   (5, D_RELEASE, 2, 0b1100), (5, D_ADMIT, 3, 0b1111),
                   (6, D_RELEASE, 3, 0b1111), (6, D_ADMIT, 4, 0b0001)]
    dec = oracle.sched_replay(oracle.device(1 << 30, queue_mode=Q_BACKFILL, **dev_kw), oracle.make_inputs(ev))
    got = [(int(d["in_index"]), int(d["kind"]), int(d["ticket"]), int(d["granule_mask"])) for d in dec]
    assert got[4:6] == [(4, D_RELEASE, 1, 0b0011), (4, D_ADMIT, 4, 0b0001)]


def test_a_workgroup_has_at_most_1024_threads():
    dev = oracle.device(1 << 30)
    ev = [("probe", 0, 1, (1, 1, 1), (1024, 1, 1)), ("probe", 1, 1, (1, 1, 1), (1025, 1, 1)),
          ("probe", 2, 1, (1, 1, 1), (32, 33, 1)), ("probe", 3, 1, (1, 1, 1), (16, 8, 8))]
    dec = oracle.sched_replay(dev, oracle.make_inputs(ev))
    assert [int(d["kind"]) for d in dec] == [D_ADMIT, D_REJECT, D_REJECT, D_ADMIT]
    assert dec[1]["code"] == dec[2]["code"] == -1          # invalid argument


def test_memory_is_hard_in_every_policy_and_exact_fit_is_admitted():
    for pol in (POL_HARD, POL_SOFT, POL_SERIAL):
        dev = oracle.device(100, policy=pol)
        ev = [("probe", 0, 100, (1, 1, 1), (64, 1, 1)), ("probe", 1, 1, (1, 1, 1), (64, 1, 1)),
              ("complete", 1)]
        dec = oracle.sched_replay(dev, oracle.make_inputs(ev))
        assert dec[0]["kind"] == D_ADMIT and dec[0]["free_bytes"] == 0     # MemReq == FreeMem fits
        assert dec[1]["kind"] == D_WAIT
        assert dec[3]["kind"] == D_ADMIT and dec[3]["in_index"] == 2


def test_all_orders_of_four_tasks_on_four_granules():
    # every arrival order and completion order: invariants hold and the set of admitted-on-arrival
    # tasks is exactly the greedy prefix-with-backfill the policy describes
    dev = oracle.device(100, n_cu=32, granule_cus=8)
    tasks = {0: (50, 128), 1: (30, 64), 2: (40, 100), 3: (20, 1)}     # mem, workgroups(256 thr)
    need = {k: -(-(-(-w // 8)) // 8) for k, (_, w) in tasks.items()}   # ceil(ceil(w/8)/8)
    for order in itertools.permutations(range(4)):
        ev = [("probe", k, tasks[k][0], (tasks[k][1], 1, 1), (256, 1, 1)) for k in order]
        free_b, free_g, expect = 100, 4, []
        for k in order:
            ok = tasks[k][0] <= free_b and need[k] <= free_g
            expect.append(ok)
            if ok:
                free_b -= tasks[k][0]
                free_g -= need[k]
        dec = oracle.sched_replay(dev, oracle.make_inputs(ev))
        assert [d["kind"] == D_ADMIT for d in dec] == expect
        for comp in itertools.permutations(range(1, 5)):
            full = ev + [("complete", t) for t in comp] * 2
            d2 = oracle.sched_replay(dev, oracle.make_inputs(full))
            assert sum(1 for d in d2 if d["kind"] == D_ADMIT) == 4
            assert sum(1 for d in d2 if d["kind"] == D_RELEASE) == 4
            assert d2[-1]["free_bytes"] == 100 or any(
                d["kind"] == D_RELEASE and d["free_bytes"] == 100 for d in d2)


def test_buddy_blocks_alignment_rounding_and_resident_limit():
    """Hand-worked: 8 granules (64 CUs), 256-thread workgroups (8 per CU, 64 per granule).
      t1 wants 3 granules -> block of 4 at [0,4).            free map 11110000
      t2 wants 1          -> [4,5).                           free map 11100000
      t3 wants 2          -> lowest aligned free pair [6,8) ([4,6) is broken by t2).  free 00100000
      t4 wants 2          -> no aligned pair left (only granule 5) -> waits
      t5 wants 1          -> [5,6) (backfill)                 free 00000000
      complete t2         -> granule 4 free; t4 still has no pair ([4,6) half busy) -> keeps waiting
      complete t5         -> [4,6) free -> t4 admitted there
    and with max_running = 2 the third task must wait although granules are free."""
    dev = oracle.device(1 << 30, n_cu=64, granule_cus=8)
    wg = lambda g: (64 * g, 1, 1)
    ev = [("probe", 1, 1, wg(3), (256, 1, 1)), ("probe", 2, 1, wg(1), (256, 1, 1)),
          ("probe", 3, 1, wg(2), (256, 1, 1)), ("probe", 4, 1, wg(2), (256, 1, 1)),
          ("probe", 5, 1, wg(1), (256, 1, 1)), ("complete", 2), ("complete", 5)]
    dec = oracle.sched_replay(dev, oracle.make_inputs(ev))
    got = [(int(d["in_index"]), int(d["kind"]), int(d["ticket"]), int(d["granule_mask"]), int(d["free_granules"]))
           for d in dec]
    assert got == [(0, D_ADMIT, 1, 0x0F, 0xF0), (1, D_ADMIT, 2, 0x10, 0xE0), (2, D_ADMIT, 3, 0xC0, 0x20),
                   (3, D_WAIT, 4, 0, 0x20), (4, D_ADMIT, 5, 0x20, 0x00),
                   (5, D_RELEASE, 2, 0x10, 0x10), (6, D_RELEASE, 5, 0x20, 0x30), (6, D_ADMIT, 4, 0x30, 0x00)]
    assert [int(d["demand"]) for d in dec[:5]] == [3, 1, 2, 2, 1]
    dev2 = oracle.device(1 << 30, n_cu=64, granule_cus=8, max_running=2)
    dec2 = oracle.sched_replay(dev2, oracle.make_inputs(ev[:3] + [("complete", 1)]))
    assert [int(d["kind"]) for d in dec2] == [D_ADMIT, D_ADMIT, D_WAIT, D_RELEASE, D_ADMIT]
    assert int(dec2[4]["ticket"]) == 3 and int(dec2[4]["granule_mask"]) == 0x03   # lowest aligned pair now free


def test_cg_ratio_ignores_memory_and_reports_the_crash():
    # Sec. IV's CG baseline: up to `ratio` jobs share the device, memory is never consulted, so
    # the job that does not fit at the moment it is let in is the one that dies.
    dev = oracle.device(1000, policy=POL_CG, max_running=2)
    g, b = (4, 1, 1), (64, 1, 1)
    ev = [("probe", 1, 600, g, b),      # t1 in, 400 free
          ("probe", 2, 600, g, b),      # below the ratio, does not fit -> out of memory, gone
          ("probe", 3, 300, g, b),      # t3 in, 100 free, ratio reached
          ("probe", 4, 500, g, b),      # t4 waits for a slot, not for memory
          ("probe", 5, 50, g, b),       # t5 waits behind it
          ("complete", 3),              # slot free, 400 bytes free: t4 (500) dies, t5 gets in
          ("complete", 2),              # the dead job's ticket is unknown
          ("complete", 1), ("complete", 5)]
    dec = oracle.sched_replay(dev, oracle.make_inputs(ev))
    got = [(int(d["in_index"]), int(d["kind"]), int(d["ticket"]), int(d["code"]), int(d["free_bytes"])) for d in dec]
    E_OOM, E_UNKNOWN = -8, -3
    assert got == [(0, D_ADMIT, 1, 0, 400), (1, D_REJECT, 2, E_OOM, 400), (2, D_ADMIT, 3, 0, 100),
                   (3, D_WAIT, 4, 0, 100), (4, D_WAIT, 5, 0, 100),
                   (5, D_RELEASE, 3, 0, 400), (5, D_REJECT, 4, E_OOM, 400), (5, D_ADMIT, 5, 0, 350),
                   (6, D_REJECT, 0, E_UNKNOWN, 350),
                   (7, D_RELEASE, 1, 0, 950), (8, D_RELEASE, 5, 0, 1000)]
    # every admitted job shares the whole device
    assert all(d["granule_mask"] == 0xFFFFFFFF for d in dec if d["kind"] == D_ADMIT)
    # with unbounded memory CG never rejects and never holds more than `ratio` jobs
    dev = oracle.device(1 << 40, policy=POL_CG, max_running=3)
    ev = [("probe", i, 1000, g, b) for i in range(1, 9)] + [("complete", i) for i in range(1, 9)]
    dec = oracle.sched_replay(dev, oracle.make_inputs(ev))
    assert (dec["kind"] == D_REJECT).sum() == 0 and (dec["kind"] == D_ADMIT).sum() == 8
    running = 0
    for d in dec:
        running += int(d["kind"] == D_ADMIT) - int(d["kind"] == D_RELEASE)
        assert running <= 3


def test_grow_is_granted_only_from_free_bytes_and_returns_with_the_task():
    dev = oracle.device(1000)
    g, b = (4, 1, 1), (64, 1, 1)
    ev = [("probe", 1, 400, g, b),      # t1 in, 600 free
          ("probe", 2, 700, g, b),      # t2 waits for memory
          ("grow", 1, 500),             # 500 <= 600: granted, 100 free
          ("grow", 1, 101),             # refused, nothing changes
          ("grow", 2, 1),               # a queued task cannot grow
          ("grow", 9, 1),               # unknown ticket
          ("grow", 1, 100),             # exact fit, 0 free
          ("complete", 1),              # the whole grown footprint (1000) comes back; t2 gets in
          ("complete", 2)]
    dec = oracle.sched_replay(dev, oracle.make_inputs(ev))
    got = [(int(d["in_index"]), int(d["kind"]), int(d["ticket"]), int(d["code"]), int(d["free_bytes"])) for d in dec]
    assert got == [(0, D_ADMIT, 1, 0, 600), (1, D_WAIT, 2, 0, 600), (2, D_GROWN, 1, 0, 100),
                   (3, D_REJECT, 1, -5, 100), (4, D_REJECT, 2, -4, 100), (5, D_REJECT, 0, -3, 100),
                   (6, D_GROWN, 1, 0, 0), (7, D_RELEASE, 1, 0, 1000), (7, D_ADMIT, 2, 0, 300),
                   (8, D_RELEASE, 2, 0, 1000)]


def test_probe_formulas_match_stated_footprints():
    import ctypes as C
    out = (C.c_uint64 * 7)()
    oracle.lib().orc_jacobi_probe(C.c_uint64(16384), C.c_uint64(4), out)
    assert out[0] == 2 * 2 ** 30                     # "about 2 GiB" per Jacobi 16384^2 task
    assert out[1] == 34304 and out[4] == 256           # 67 x 2048 windows, four per workgroup
    oracle.lib().orc_jacobi_probe(C.c_uint64(16384), C.c_uint64(50), out)
    assert out[0] == 2 * 2 ** 30 and out[1] == 7080    # 8 launches of 6-7 sweeps: 69 strips of 240 columns x 410 runs of 40 rows
    oracle.lib().orc_gemm_f32_probe(C.c_uint64(32768), C.c_uint64(32768), C.c_uint64(32768), out)
    assert out[0] == 12 * 2 ** 30                    # "about 12 GiB" per GEMM 32768^3 task
    assert out[1] == 128 * 128 and out[4] == 256       # 256 x 256 tiles, four waves each
    oracle.lib().orc_jacobi_probe(C.c_uint64(512), C.c_uint64(20), out)
    assert out[0] == 2 * 512 * 512 * 4 and out[1] == 48   # 3 x 64 windows, four per workgroup
    oracle.lib().orc_gemm_f32_probe(C.c_uint64(256), C.c_uint64(256), C.c_uint64(256), out)
    assert out[0] == 768 * 1024 and out[1] == 16 and out[4] == 256   # 4 x 4 tiles of 64 x 64 (too few 128 x 128 ones)
