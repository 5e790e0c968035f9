"""Pins for the CPU oracle's allocator, lane assignment and scheduler.

None of these tests compares the oracle with itself: each one checks it against
numbers worked by hand from the paper (tests/golden), against the safety
condition, or against an independent brute-force model written here.
"""
import itertools
import os
import random

import numpy as np
import pytest

from oracle import pool as op

GOLD = os.path.join(os.path.dirname(__file__), "golden")
MiB, GB = 1 << 20, 10 ** 9


def rows(name):
    with open(os.path.join(GOLD, name)) as f:
        return [[int(x) for x in ln.split()] for ln in f if ln.strip() and ln[0] != '#']


# ------------------------------------------------------------------ worked examples
def test_deadlock_example_shares_one_lane():
    (C, P, E, la, lb, nl), = rows("deadlock_example.txt")
    p = op.Pool(C * GB, granule=1000)
    sa, a = p.job_arrive(P * GB, E * GB)
    sb, b = p.job_arrive(P * GB, E * GB)
    assert (sa, sb) == (op.OK, op.OK)
    assert (p.jobs[a].lane, p.jobs[b].lane, len(p.lanes)) == (la, lb, nl)
    p.check_invariants()
    # serialized: a round runs exactly one of them
    p.set_pending(a, 5), p.set_pending(b, 5)
    assert all(len(p.schedule_iteration()) == 1 for _ in range(4))


def test_workload1_layout_matches_hand_trace():
    p = op.Pool(4 * MiB, granule=256, policy=op.RR)
    for _ in range(4):
        st, _ = p.job_arrive(512 * 1024, MiB, 0, 8)
        assert st == op.OK
    for job, lane, base, size, off in rows("workload1_layout.txt"):
        j = p.jobs[job]
        assert (j.lane, p.lane_base(j.lane), p.lane_by_id(j.lane).size, j.off) == \
               (lane, base, size, off)
    # round-robin inside each lane: rounds alternate {0,1} and {2,3}
    seq = [p.schedule_iteration() for _ in range(16)]
    assert seq == [[(0, 0), (1, 1)], [(2, 0), (3, 1)]] * 8
    assert all(j.pending == 0 and j.served == 8 for j in p.jobs)
    assert p.schedule_iteration() == []


def test_never_fits_and_queueing():
    p = op.Pool(1000, granule=10)
    assert p.job_arrive(600, 500)[0] == op.ENEVER          # cannot run even alone
    assert p.job_arrive(0, 10)[0] == op.EINVAL
    assert p.job_arrive(300, 300)[0] == op.OK               # lane 0
    st, q = p.job_arrive(300, 600)                          # 300+300 + 600 > 1000 in any branch
    assert st == op.IS_QUEUED and p.Q == [q]
    p.check_invariants()
    assert p.job_finish(0) == op.OK                         # lane 0 goes away -> queue retried
    assert p.jobs[q].state == op.RESIDENT and p.Q == []
    p.check_invariants()


def test_findlane_prefers_new_then_best_match_then_grow():
    p = op.Pool(100, granule=1)
    _, a = p.job_arrive(5, 30)          # new lane 0 (30)
    _, b = p.job_arrive(5, 20)          # new lane 1 (20): 10+50 <= 100
    assert [l.size for l in p.lanes] == [30, 20]
    _, c = p.job_arrive(5, 18)          # new lane 2 (18): 15 + 68 = 83
    _, d = p.job_arrive(5, 19)          # new would be 20+68+19 = 107 > 100 -> best match
    assert p.jobs[d].lane == 1          # slack 1 in lane 1 (20) beats slack 11 in lane 0
    _, e = p.job_arrive(2, 25)          # 22+68 = 90: fits lane 0 only
    assert p.jobs[e].lane == 0
    _, f = p.job_arrive(1, 31)          # nothing fits 31; grow smallest lane first:
    # lane 2 (18) -> 23 + 68 - 18 + 31 = 104 > 100; lane 1 (20) -> 102 > 100; lane 0 (30) -> 92
    assert p.jobs[f].lane == 0 and p.lane_by_id(0).size == 31
    p.check_invariants()


def test_grow_picks_smallest_feasible_lane():
    p = op.Pool(100, granule=1)
    p.job_arrive(10, 20)
    p.job_arrive(10, 30)
    _, c = p.job_arrive(10, 35)         # new: 30+50+35 = 115; no lane >= 35; grow lane 0: 30+50-20+35 = 95
    assert p.jobs[c].lane == 0 and [l.size for l in p.lanes] == [35, 30]
    p.check_invariants()


def test_best_match_tie_goes_to_lane_with_fewer_jobs_then_oldest():
    p = op.Pool(64, granule=1, max_lanes=2)
    for _ in range(2):
        p.job_arrive(1, 10)
    assert [p.job_arrive(1, 10)[1] for _ in range(3)] == [2, 3, 4]
    assert [p.jobs[i].lane for i in range(5)] == [0, 1, 0, 1, 0]


def test_lane_lives_until_last_job_leaves_and_neighbours_slide_for_free():
    mem = np.zeros(100, np.uint8)
    p = op.Pool(100, granule=1, mem=mem, max_lanes=3)
    _, a = p.job_arrive(5, 20)          # lane 0 = [80,100)
    _, b = p.job_arrive(5, 10)          # lane 1 = [70,80)
    _, c = p.job_arrive(5, 20)          # lane 2 = [50,70)
    _, d = p.job_arrive(5, 20)          # three lanes is the cap -> shares lane 0 or 2 (slack 0, one job each): oldest
    assert p.jobs[d].lane == 0 and p.lane_by_id(0).ref == 2
    assert [p.lane_base(i) for i in (0, 1, 2)] == [80, 70, 50]
    p.job_finish(a)
    assert len(p.lanes) == 3            # d still holds lane 0
    p.job_finish(b)                     # lane 1 disappears, lane 2 slides up by 10
    assert [l.id for l in p.lanes] == [0, 2] and p.lane_base(2) == 60
    assert p.stats['bytes_d2d'] == 0 and p.stats['moves'] == 0     # nothing was copied
    assert p.stats['lanes_deleted'] == 1 and p.stats['lanes_moved'] == 1
    p.check_invariants()


def test_queued_job_admitted_when_a_lane_disappears():
    p = op.Pool(100, granule=1)
    _, a = p.job_arrive(10, 40)
    _, b = p.job_arrive(10, 30)
    st, c = p.job_arrive(30, 35)        # new 50+70+35; use lane0: 50+70=120 > 100; queued
    assert st == op.IS_QUEUED
    p.job_finish(b)                     # lane 1 gone: 40 + 40 + 35 > 100, lane 0: 40+40 <= 100
    assert p.jobs[c].state == op.RESIDENT and p.jobs[c].lane == 0
    p.check_invariants()


# ------------------------------------------------------------------ brute force
def independent_feasible(C, A, max_lanes, resident_P, lanes, P, E):
    """Is there ANY single action (open / join / grow one lane) after which the
    safety condition  sum P + sum L <= C,  L >= E  holds?  Written directly from
    the safety condition, not from FindLane."""
    SP = sum(resident_P) + P
    if (max_lanes == 0 or len(lanes) < max_lanes) and SP + sum(lanes) + E <= C:
        return True
    for i, L in enumerate(lanes):
        newL = max(L, E)
        if SP + sum(lanes) - L + newL <= C:
            return True
    return False


def interleavings(n):
    """All event orders of n jobs: arrivals in job order, each finish after its arrival."""
    def rec(seq, arrived, finished):
        if len(seq) == 2 * n:
            yield list(seq)
            return
        if arrived < n:
            yield from rec(seq + ["a"], arrived + 1, finished)
        for j in range(arrived):
            if j not in finished:
                yield from rec(seq + [j], arrived, finished | {j})
    return rec([], 0, frozenset())


@pytest.mark.parametrize("max_lanes", [0, 2])
def test_bruteforce_tiny_pools(max_lanes):
    """Pool of 16 granules: every (P, E) combination of three jobs from a small
    set, under every arrive/finish interleaving, plus four-job scripts."""
    C, A = 16, 1
    sizes = [(1, 2), (2, 5), (3, 3), (1, 8), (4, 7), (6, 9)]
    scripts3 = list(interleavings(3))
    assert len(scripts3) == 15       # 6! / (2^3 * 3!)
    scripts4 = [["a", "a", "a", "a", 0, 2, 1, 3], ["a", "a", 0, "a", "a", 1, 3, 2],
                ["a", "a", "a", 1, "a", 0, 3, 2], ["a", 0, "a", "a", 2, "a", 1, 3]]
    cases = [(c, s) for c in itertools.product(range(len(sizes)), repeat=3) for s in scripts3]
    cases += [(c, s) for c in itertools.product(range(len(sizes)), repeat=4) for s in scripts4]
    checked = 0
    for combo, script in cases:
        p = op.Pool(C, granule=A, max_lanes=max_lanes, policy=op.PACK,
                    mem=np.zeros(C, np.uint8))
        content, nxt = {}, 0
        for ev in script:
            if ev == "a":
                P, E = sizes[combo[nxt]]
                nxt += 1
                p.job_arrive(P, E, 0, 3)
            else:
                p.job_finish(ev)
                content.pop(ev, None)
            # give newly admitted jobs recognisable bytes
            for j in p.jobs:
                if j.state == op.RESIDENT and j.id not in content:
                    content[j.id] = np.full(j.P, 10 + j.id, np.uint8)
                    p.mem[j.off:j.off + j.P] = content[j.id]
            p.check_invariants()
            # persistent bytes survive whatever compaction happened
            for j in p.jobs:
                if j.state == op.RESIDENT:
                    assert (p.mem[j.off:j.off + j.P] == content[j.id]).all()
            # nobody waits while a feasible action exists
            for q in p.Q:
                j = p.jobs[q]
                assert not independent_feasible(
                    C, A, max_lanes, [r.P for r in p.resident()],
                    [l.size for l in p.lanes], j.P, j.E)
            checked += 1
    assert checked > 50000


def test_random_event_sequences_keep_invariants_and_bytes():
    for seed in range(30):
        rnd = random.Random(seed)
        C = 4096
        p = op.Pool(C, granule=16, max_lanes=rnd.choice([0, 3, 6]),
                    policy=rnd.choice([op.RR, op.PACK, op.PRIORITY, op.FIFO]),
                    mem=np.zeros(C, np.uint8))
        content = {}
        for step in range(200):
            r = rnd.random()
            alive = [j.id for j in p.jobs if j.state != op.DONE]
            if r < 0.45 or not alive:
                p.job_arrive(rnd.randint(1, 700), rnd.randint(1, 900), rnd.randint(0, 3),
                             rnd.randint(1, 20))
            elif r < 0.8:
                jid = rnd.choice(alive)
                p.job_finish(jid)
                content.pop(jid, None)
            elif r < 0.9:
                p.schedule_iteration()
            else:
                jid = rnd.choice(alive)
                if p.jobs[jid].state == op.RESIDENT:
                    assert p.switch_out(jid) == op.OK
                elif p.jobs[jid].state == op.EVICTED:
                    assert p.switch_in(jid) in (op.OK, op.ENOMEM)
            for j in p.jobs:
                if j.state == op.RESIDENT and j.id not in content:
                    content[j.id] = np.frombuffer(random.Random(seed * 1000 + j.id)
                                                  .randbytes(j.P), np.uint8).copy()
                    p.mem[j.off:j.off + j.P] = content[j.id]
            p.check_invariants()
            for j in p.jobs:
                if j.state == op.RESIDENT:
                    assert (p.mem[j.off:j.off + j.P] == content[j.id]).all(), (seed, step, j.id)


# ------------------------------------------------------------------ compaction
def test_compaction_closed_form_and_idempotent():
    C = 1000
    mem = np.arange(C, dtype=np.uint32).astype(np.uint8)
    p = op.Pool(C, granule=10, mem=mem, max_lanes=1)
    ids = [p.job_arrive(s, 50)[1] for s in (95, 41, 200, 7, 120)]   # rounded 100,50,200,10,120
    assert [p.jobs[i].off for i in ids] == [0, 100, 150, 350, 360]
    for i in ids:
        j = p.jobs[i]
        mem[j.off:j.off + j.P] = 100 + i
    p.job_finish(ids[1])
    p.job_finish(ids[3])
    before = {i: mem[p.jobs[i].off:p.jobs[i].off + p.jobs[i].P].copy() for i in (0, 2, 4)}
    plan = p.compact()
    # exclusive prefix sum of rounded sizes 100, 200, 120; block 0 does not move
    assert plan == [(150, 100, 200), (360, 300, 120)]
    assert [p.jobs[i].off for i in (0, 2, 4)] == [0, 100, 300]
    for i in (0, 2, 4):
        j = p.jobs[i]
        assert (mem[j.off:j.off + j.P] == before[i]).all()
    assert p.holes(p.floor()) == [(420, p.floor() - 420)]          # a single free range
    assert p.compact() == []                                        # idempotent
    assert p.stats['bytes_d2d'] == 320 and p.stats['moves'] == 2


def test_compaction_with_overlapping_source_and_destination():
    C = 64
    mem = np.zeros(C, np.uint8)
    p = op.Pool(C, granule=1, mem=mem, max_lanes=1)
    a = p.job_arrive(2, 4)[1]
    b = p.job_arrive(40, 4)[1]
    mem[2:42] = np.arange(1, 41)
    p.job_finish(a)
    assert p.compact() == [(2, 0, 40)]       # shift (2) far smaller than the block (40)
    assert (mem[0:40] == np.arange(1, 41)).all()


def test_allocation_triggers_compaction_only_when_fragmented():
    p = op.Pool(100, granule=1, max_lanes=1, mem=np.zeros(100, np.uint8))
    a = p.job_arrive(20, 10)[1]
    b = p.job_arrive(20, 10)[1]
    c = p.job_arrive(20, 10)[1]
    p.job_finish(a)
    p.job_finish(c)                          # free: [0,20) and [40,90)
    assert p.stats['compactions'] == 0
    d = p.job_arrive(45, 10)[1]              # fits the upper hole: no compaction
    assert p.jobs[d].off == 40 and p.stats['compactions'] == 0
    p.job_finish(d)
    e = p.job_arrive(60, 10)[1]              # 70 free in total, largest hole 50 -> compaction
    assert p.stats['compactions'] == 1 and p.jobs[b].off == 0 and p.jobs[e].off == 20


def test_new_lane_pushes_persistent_blocks_below_the_new_floor():
    p = op.Pool(100, granule=1, mem=np.zeros(100, np.uint8))
    a = p.job_arrive(30, 10)[1]              # lane 0 = [90,100), block [0,30)
    b = p.job_arrive(30, 10)[1]              # lane 1 = [80,90),  block [30,60)
    p.mem[30:60] = 7
    p.job_finish(a)                          # lane 0 gone; lane 1 = [90,100); hole [0,30)
    c = p.job_arrive(10, 50)[1]              # new lane [40,90): block b reaches 60 > 40 -> compact first
    assert p.jobs[b].off == 0 and p.jobs[c].off == 30 and (p.mem[0:30] == 7).all()
    p.check_invariants()


# ------------------------------------------------------------------ switching
def test_switch_out_in_is_byte_exact_and_first_fit():
    C = 4 * 1024
    mem = np.zeros(C, np.uint8)
    p = op.Pool(C, granule=256, mem=mem, max_lanes=1)
    ids = [p.job_arrive(512, 256)[1] for _ in range(4)]
    rng = np.random.default_rng(0)
    data = {i: rng.integers(0, 256, 512, dtype=np.uint8) for i in ids}
    for i in ids:
        mem[p.jobs[i].off:p.jobs[i].off + 512] = data[i]
    assert p.switch_out(2) == op.OK and p.jobs[2].state == op.EVICTED
    assert p.switch_out(2) == op.ENOTRESIDENT
    mem[1024:1536] = 0xEE                     # the freed bytes may be reused by anyone
    assert p.switch_in(2) == op.OK and p.jobs[2].off == 1024     # same hole again
    for i in ids:
        assert (mem[p.jobs[i].off:p.jobs[i].off + 512] == data[i]).all()
    assert p.stats['bytes_d2h'] == 512 and p.stats['bytes_h2d'] == 512


def test_priority_admission_evicts_and_restores():
    """Scaled-down preemption scenario: a long low-priority job with a large
    persistent state and a short urgent job that does not fit beside it."""
    C = 23 * 1024
    mem = np.zeros(C, np.uint8)
    p = op.Pool(C, granule=256, policy=op.PRIORITY, mem=mem)
    _, low = p.job_arrive(20 * 1024, 2 * 1024, priority=0, pending=10 ** 6)
    state = np.random.default_rng(3).integers(0, 256, 20 * 1024, dtype=np.uint8)
    mem[0:20 * 1024] = state
    st, high = p.job_arrive(2 * 1024, 2 * 1024, priority=5, pending=10)
    assert st == op.OK
    assert p.jobs[low].state == op.EVICTED and p.jobs[low].auto_evicted
    mem[:] = 0x55                                                   # urgent job scribbles anywhere
    assert [j for j, _ in p.schedule_iteration()] == [high]         # the evicted job cannot run
    p.check_invariants()
    p.job_finish(high)
    assert p.jobs[low].state == op.RESIDENT
    off = p.jobs[low].off
    assert (mem[off:off + 20 * 1024] == state).all()
    assert p.stats['bytes_d2h'] == 20 * 1024 == p.stats['bytes_h2d']
    # an equal-priority arrival never evicts
    st, same = p.job_arrive(2 * 1024, 2 * 1024, priority=0, pending=1)
    assert st == op.IS_QUEUED and p.jobs[low].state == op.RESIDENT


def test_priority_eviction_is_skipped_when_it_cannot_help():
    """Nothing is evicted for a request that would not fit even then: the room is
    held by a job of the same priority, which is never a victim."""
    p = op.Pool(100, granule=1, policy=op.PRIORITY)
    _, a = p.job_arrive(30, 40, priority=9, pending=5)
    _, low = p.job_arrive(10, 10, priority=0, pending=5)
    st, b = p.job_arrive(35, 40, priority=9, pending=5)   # without low: 30+35 + lane 40 = 105 > 100
    assert st == op.IS_QUEUED and p.stats['evictions'] == 0
    assert p.jobs[low].state == op.RESIDENT and p.jobs[a].state == op.RESIDENT
    p.check_invariants()


def test_priority_job_that_fits_alone_is_admitted_whatever_runs():
    """Section 4.2: the higher-priority job is admitted as long as it could run
    alone (P + E <= C), regardless of the jobs already running.  The lane of
    the job evicted for it must not stand in the way: a lane with no resident
    job is parked (reserves nothing) until one of its jobs returns."""
    mem = np.zeros(100, np.uint8)
    p = op.Pool(100, granule=1, policy=op.PRIORITY, mem=mem)
    _, low = p.job_arrive(10, 60, priority=0, pending=50)
    mem[0:10] = np.arange(1, 11)
    assert p.lane_base(0) == 40
    st, high = p.job_arrive(50, 45, priority=9, pending=5)     # 50 + 45 = 95 <= 100
    assert st == op.OK and p.jobs[low].state == op.EVICTED and p.jobs[low].auto_evicted
    assert [l.id for l in p.lanes] == [0, 1] and p.parked(p.lanes[0]) and not p.parked(p.lanes[1])
    assert p.sum_L() == 45 and p.floor() == 55 and p.lane_base(1) == 55 and p.jobs[high].off == 0
    kinds = [e[0] for e in p.events]
    assert kinds[-4:] == [op.EV_EVICT, op.EV_LANE_PARK, op.EV_LANE_NEW, op.EV_ADMIT]
    p.check_invariants()
    mem[:] = 0x77
    assert p.schedule_iteration() == [(high, 1)]
    assert p.switch_in(low) == op.ENOMEM                       # 50 + 10 + 45 + 60 > 100
    p.job_finish(high)
    assert p.jobs[low].state == op.RESIDENT and p.jobs[low].off == 0
    assert (mem[0:10] == np.arange(1, 11)).all()
    assert not p.parked(p.lanes[0]) and p.lane_base(0) == 40 and p.sum_L() == 60
    assert p.events[-2] == (op.EV_LANE_UNPARK, 0, 60) and p.events[-1] == (op.EV_RESTORE, low, 0)
    p.check_invariants()


def test_parked_lane_rules():
    # a lane is parked only when ALL its jobs are evicted, and any restore unparks it
    p = op.Pool(100, granule=1, max_lanes=2, policy=op.RR)
    a = p.job_arrive(10, 30)[1]
    b = p.job_arrive(10, 20)[1]                 # lane 1
    c = p.job_arrive(10, 30)[1]                 # shares lane 0 (exact fit)
    assert [p.jobs[x].lane for x in (a, b, c)] == [0, 1, 0]
    assert p.switch_out(a) == op.OK and p.sum_L() == 50 and p.lane_base(1) == 50
    assert p.switch_out(c) == op.OK and p.sum_L() == 20 and p.lane_base(1) == 80   # lane 1 slid up
    p.check_invariants()
    # parked lanes are invisible to FindLane: not shared, not grown, not counted
    d = p.job_arrive(10, 30)[1]
    assert p.jobs[d].lane == 2 and p.lane_base(2) == 50
    # the cap counts lanes that hold memory: lane 0 cannot come back while two others do
    assert p.switch_in(a) == op.ENOMEM
    p.job_finish(b)
    assert p.switch_in(a) == op.OK and p.lane_base(0) == 70 and p.lane_base(2) == 40
    assert p.jobs[c].state == op.EVICTED        # its lane is back, the job itself is not
    p.check_invariants()
    # a parked lane whose last job finishes is deleted without any slide
    q = op.Pool(100, granule=1, policy=op.RR)
    x = q.job_arrive(10, 30)[1]
    y = q.job_arrive(10, 20)[1]
    q.switch_out(x)
    moved = q.stats['lanes_moved']
    q.job_finish(x)
    assert [l.id for l in q.lanes] == [1] and q.stats['lanes_moved'] == moved and q.lane_base(1) == 80
    q.check_invariants()


def test_strictly_most_urgent_arrival_is_always_admitted_at_once():
    """Property behind Section 4.2, on random pools: under PRIORITY an arrival
    whose priority is above every other job's and whose P + E <= C is resident
    when job_arrive returns, whatever was running."""
    rng = np.random.default_rng(11)
    for trial in range(200):
        C = int(rng.integers(40, 200))
        p = op.Pool(C, granule=1, policy=op.PRIORITY, max_lanes=int(rng.integers(0, 4)))
        for _ in range(int(rng.integers(1, 8))):
            p.job_arrive(int(rng.integers(1, C // 2)), int(rng.integers(1, C // 2)),
                         priority=int(rng.integers(0, 5)), pending=3)
            p.check_invariants()
        live = [j for j in p.jobs if j.state == op.RESIDENT]
        for j in live[:int(rng.integers(0, 3))]:
            p.job_finish(j.id)
        P = int(rng.integers(1, C))
        E = int(rng.integers(1, C - P + 1))
        st, u = p.job_arrive(P, E, priority=9, pending=3)
        assert st == op.OK, (trial, C, P, E)
        p.check_invariants()
        p.job_finish(u)
        p.check_invariants()


# ------------------------------------------------------------------ scheduling
def test_fair_share_follows_arrivals_and_departures():
    """Section 5.1.2, fair sharing: with n equal jobs in one lane each gets 1/n of
    the iterations, and the share changes right when a job arrives or leaves.
    Only the public calls are used: the oracle's state is never edited."""
    p = op.Pool(1000, granule=1, max_lanes=1, policy=op.RR)

    def run(rounds):
        out = []
        for _ in range(rounds):
            (j, _), = p.schedule_iteration()
            out.append(j)
        return out
    a = p.job_arrive(10, 100, 0, 10 ** 6)[1]
    assert run(6) == [a] * 6                                  # share 1
    b = p.job_arrive(10, 100, 0, 10 ** 6)[1]
    got = run(6)
    assert got.count(a) == 3 and got.count(b) == 3            # halved at once, not after a catch-up burst
    assert set(got[:2]) == {a, b}                             # ... within the very first two rounds
    c = p.job_arrive(10, 100, 0, 10 ** 6)[1]
    got = run(9)
    assert [got.count(x) for x in (a, b, c)] == [3, 3, 3]     # a third each
    assert set(got[:3]) == {a, b, c}
    p.job_finish(c)
    got = run(6)
    assert got.count(a) == 3 and got.count(b) == 3            # the reverse when jobs leave
    p.job_finish(b)
    assert run(4) == [a] * 4


def test_fair_newcomer_starts_level_with_the_jobs_it_competes_with():
    """Reading of Section 4.3 against Section 5.1.2: a job that enters a lane
    starts at the least attained service among the lane's runnable jobs (not at
    zero), else among its resident jobs; zero in an empty lane."""
    p = op.Pool(1000, granule=1, max_lanes=1, policy=op.RR)
    a = p.job_arrive(10, 100, 0, 100)[1]
    b = p.job_arrive(10, 100, 0, 100)[1]
    for _ in range(10):
        p.schedule_iteration()
    assert (p.jobs[a].attained, p.jobs[b].attained) == (5, 5)
    p.set_pending(b, 0)                       # b idles; a runs alone
    for _ in range(4):
        p.schedule_iteration()
    assert (p.jobs[a].attained, p.jobs[b].attained) == (9, 5)
    c = p.job_arrive(10, 100, 0, 100)[1]      # competes with a only: starts at 9, not at b's 5
    assert p.jobs[c].attained == 9 and p.jobs[c].served == 0
    p.set_pending(a, 0)
    d = p.job_arrive(10, 100, 0, 100)[1]      # runnable: c (9) -> 9
    assert p.jobs[d].attained == 9
    p.set_pending(c, 0), p.set_pending(d, 0)
    e = p.job_arrive(10, 100, 0, 100)[1]      # nobody runnable: least among the resident jobs
    assert p.jobs[e].attained == 5
    # costs: the level is in the same unit as the service it is compared with
    q = op.Pool(1000, granule=1, max_lanes=1, policy=op.RR)
    x = q.job_arrive(10, 100, 0, 100)[1]
    q.set_cost(x, 7)
    for _ in range(3):
        q.schedule_iteration()
    y = q.job_arrive(10, 100, 0, 100)[1]
    assert q.jobs[y].attained == 21
    # a queued job gets its level when it is admitted, not when it arrives
    r = op.Pool(100, granule=1, max_lanes=1, policy=op.RR)
    u = r.job_arrive(40, 10, 0, 100)[1]
    v = r.job_arrive(40, 10, 0, 100)[1]
    w = r.job_arrive(40, 10, 0, 100)[1]
    assert r.jobs[w].state == op.QUEUED
    for _ in range(6):
        r.schedule_iteration()
    r.job_finish(u)
    assert r.jobs[w].state == op.RESIDENT and r.jobs[w].attained == r.jobs[v].attained == 3


def test_fair_strict_rotation_for_equal_jobs():
    p = op.Pool(1000, granule=1, max_lanes=1, policy=op.RR)
    ids = [p.job_arrive(10, 100, 0, 100)[1] for _ in range(3)]
    seq = [p.schedule_iteration()[0][0] for _ in range(9)]
    assert seq == ids * 3


def test_srtf_order_relations():
    """Section 5.1.2, SRTF trace: a newly arrived shorter job stops the long
    background job at once; of two waiting jobs the shorter runs first even if
    it came later; a still shorter arrival preempts the running one; the
    background job runs only when nothing shorter exists."""
    p = op.Pool(10000, granule=1, max_lanes=1, policy=op.PRIORITY)
    j0 = p.job_arrive(10, 100, 0, 1000)[1]
    run = lambda: p.schedule_iteration()[0][0]
    assert [run() for _ in range(3)] == [j0] * 3
    j1 = p.job_arrive(10, 100, 0, 4)[1]
    assert run() == j1                         # background job stopped immediately
    j2 = p.job_arrive(10, 100, 0, 20)[1]       # arrives before j3 ...
    j3 = p.job_arrive(10, 100, 0, 6)[1]        # ... but j3 is shorter
    order = [run() for _ in range(3 + 6)]
    assert order == [j1] * 3 + [j3] * 6
    j4 = j2
    assert [run() for _ in range(5)] == [j4] * 5
    j5 = p.job_arrive(10, 100, 0, 3)[1]        # shorter than what is left of j4 (15)
    assert [run() for _ in range(3)] == [j5] * 3
    assert [run() for _ in range(15)] == [j4] * 15
    assert run() == j0                         # only now the background job


def test_priority_beats_remaining_time():
    p = op.Pool(10000, granule=1, max_lanes=1, policy=op.PRIORITY)
    a = p.job_arrive(10, 100, priority=1, pending=100)[1]
    b = p.job_arrive(10, 100, priority=0, pending=2)[1]
    assert [p.schedule_iteration()[0][0] for _ in range(3)] == [a, a, a]


def test_pack_runs_every_lane_and_fifo_runs_one_job():
    p = op.Pool(1000, granule=1, policy=op.PACK)
    ids = [p.job_arrive(10, 50, 0, 2)[1] for _ in range(5)]
    assert len(p.lanes) == 5
    assert p.schedule_iteration() == [(i, i) for i in ids]
    p.set_pending(ids[2], 0)                   # a model with no request is skipped
    assert [j for j, _ in p.schedule_iteration()] == [0, 1, 3, 4]
    q = op.Pool(1000, granule=1, policy=op.FIFO)
    ids = [q.job_arrive(10, 50, 0, 2)[1] for _ in range(3)]
    assert [q.schedule_iteration() for _ in range(7)] == \
        [[(0, 0)], [(0, 0)], [(1, 1)], [(1, 1)], [(2, 2)], [(2, 2)], []]


def test_lane_shrinks_to_largest_remaining_peak_when_asked():
    """Section 3.3.2 defines L_j = max E_i over the lane's jobs.  Hand-worked:
    C = 10000, one lane shared by E = 1000, 3000, 2000; a younger lane of 2500."""
    p = op.Pool(10000, granule=1, max_lanes=2, policy=op.RR, shrink_lanes=True)
    a = p.job_arrive(500, 3000)[1]
    b = p.job_arrive(500, 2500)[1]
    c = p.job_arrive(500, 1000)[1]          # joins the lane with least slack that fits
    d = p.job_arrive(500, 2000)[1]
    la = p.jobs[a].lane
    assert p.jobs[d].lane == p.jobs[c].lane
    lanes0 = {l.id: (p.lane_base(l.id), l.size) for l in p.lanes}
    assert lanes0[la] == (7000, 3000)
    p.events.clear()
    # the largest job of a shared lane leaves: the lane falls back to the next peak
    shared = p.jobs[c].lane
    big = a if shared == la else b
    was = p.lane_by_id(shared).size
    p.job_finish(big)
    rest = max(p.jobs[j].E for j in (c, d))
    assert p.lane_by_id(shared).size == rest == 2000 < was
    assert (op.EV_LANE_SHRINK, shared, 2000) in [tuple(e) for e in p.events]
    # lanes still tile the top of the pool, in creation order, with no gap
    top = 10000
    for l in p.lanes:
        top -= l.size
        assert p.lane_base(l.id) == top
    assert top == p.floor()
    p.check_invariants()
    # without the option Algorithm 1 keeps the lane at its high-water mark
    q = op.Pool(10000, granule=1, max_lanes=2, policy=op.RR)
    ids = [q.job_arrive(500, e)[1] for e in (3000, 2500, 1000, 2000)]
    q.job_finish(ids[0] if q.jobs[ids[2]].lane == q.jobs[ids[0]].lane else ids[1])
    assert q.lane_by_id(q.jobs[ids[2]].lane).size == was


def test_lane_shrinking_frees_room_for_a_queued_job():
    p = op.Pool(10000, granule=1, max_lanes=1, policy=op.RR, shrink_lanes=True)
    a = p.job_arrive(1000, 6000)[1]
    b = p.job_arrive(1000, 1000)[1]
    st, c = p.job_arrive(5000, 1000)          # 2000 + 5000 + 6000 > C: must wait
    assert st == op.IS_QUEUED
    p.job_finish(a)                            # lane 6000 -> 1000, then the queue is served
    assert p.jobs[c].state == op.RESIDENT and p.lanes[0].size == 1000
    p.check_invariants()
    q = op.Pool(10000, granule=1, max_lanes=1, policy=op.RR)
    a = q.job_arrive(1000, 6000)[1]
    q.job_arrive(1000, 1000)
    st, c = q.job_arrive(5000, 1000)
    q.job_finish(a)                            # 1000 + 5000 + 6000 > C still
    assert q.jobs[c].state == op.QUEUED


def test_lane_shrinking_keeps_the_equality_on_random_traces():
    import random
    hits = 0
    for seed in range(20):
        rnd = random.Random(seed)
        p = op.Pool(1 << 16, granule=64, max_lanes=3, policy=op.RR, shrink_lanes=True)
        for _ in range(300):
            alive = [j.id for j in p.jobs if j.state != op.DONE]
            if rnd.random() < 0.55 or not alive:
                p.job_arrive(rnd.randint(1, 6000), rnd.randint(1, 9000), 0, 5)
            else:
                p.job_finish(rnd.choice(alive))
            p.check_invariants()               # includes L_j == max E_i for every lane
            hits += sum(1 for e in p.events if e[0] == op.EV_LANE_SHRINK)
            p.events.clear()
    assert hits > 50


# ------------------------------------------------------------------ jobs in transit
def test_held_job_is_not_runnable_and_fair_share_catches_up():
    p = op.Pool(1 << 20, granule=256, max_lanes=1, policy=op.RR)
    ids = [p.job_arrive(4096, 4096, 0, 1000)[1] for _ in range(3)]
    assert len(p.lanes) == 1
    runs = lambda n: [p.schedule_iteration()[0][0] for _ in range(n)]
    assert runs(6) == ids * 2                                   # 1/3 each
    assert p.hold(ids[1]) == op.OK
    assert runs(6) == [ids[0], ids[2]] * 3                      # 1/2 each while one is held
    p.check_invariants()
    assert p.release(ids[1]) == op.OK
    assert runs(3) == [ids[1]] * 3                              # least attained service first
    assert runs(3) == ids
    assert [p.jobs[i].served for i in ids] == [6, 6, 6]


def test_hold_error_codes_and_layout_is_untouched():
    mem = np.zeros(1 << 16, np.uint8)
    p = op.Pool(1 << 16, granule=256, mem=mem, policy=op.RR)
    a = p.job_arrive(4096, 4096, 0, 5)[1]
    b = p.job_arrive(8192, 4096, 0, 5)[1]
    before = (p.jobs[a].off, p.jobs[b].off, [(l.id, l.size) for l in p.lanes])
    assert p.hold(7) == op.EINVAL and p.release(a) == op.EINVAL
    assert p.hold(a) == op.OK and p.hold(a) == op.EBUSY
    assert p.job_finish(a) == op.EBUSY and p.switch_out(a) == op.EBUSY
    assert (p.jobs[a].off, p.jobs[b].off, [(l.id, l.size) for l in p.lanes]) == before
    assert p.switch_out(b) == op.OK and p.hold(b) == op.ENOTRESIDENT
    assert p.release(a) == op.OK and p.job_finish(a) == op.OK
    p.check_invariants()


def test_priority_admission_never_evicts_a_held_job():
    def scenario(hold_big):
        p = op.Pool(100, granule=1, policy=op.PRIORITY, max_lanes=1)
        big = p.job_arrive(50, 10, 0, 5)[1]
        small = p.job_arrive(20, 10, 0, 5)[1]             # shares the lane: 70 + 10 = 80
        if hold_big:
            p.hold(big)
        st, urgent = p.job_arrive(35, 10, 9, 5)           # needs 35 of the 20 that are free
        return p, big, small, urgent, st
    p, big, small, urgent, st = scenario(False)
    assert st == op.OK and p.jobs[big].state == op.EVICTED and p.jobs[small].state == op.RESIDENT
    p, big, small, urgent, st = scenario(True)            # the largest candidate is in transit
    assert p.jobs[big].state == op.RESIDENT
    assert st == op.OK and p.jobs[small].state == op.EVICTED      # 50 + 35 + 10 <= 100
    p.check_invariants()
    # and if the remaining candidates cannot make room, nothing is evicted
    p = op.Pool(100, granule=1, policy=op.PRIORITY, max_lanes=1)
    big = p.job_arrive(60, 10, 0, 5)[1]
    small = p.job_arrive(10, 10, 0, 5)[1]
    p.hold(big)
    st, urgent = p.job_arrive(35, 10, 9, 5)               # 60 + 35 + 10 > 100 even without small
    assert st == op.IS_QUEUED and p.jobs[small].state == op.RESIDENT
    p.check_invariants()


# ------------------------------------------------------------------ service measured in time
def test_fair_equalizes_attained_time_not_iteration_counts():
    """Two jobs share a lane; one iteration of b lasts three times one of a.  Equal
    service time means a runs three iterations for each one of b (Section 4, FAIR)."""
    p = op.Pool(1 << 20, granule=256, max_lanes=1, policy=op.RR)
    a = p.job_arrive(4096, 4096, 0, 1000)[1]
    b = p.job_arrive(4096, 4096, 0, 1000)[1]
    assert p.set_cost(b, 3) == op.OK
    seq = [p.schedule_iteration()[0][0] for _ in range(16)]
    # attained (a, b): (0,0) a, (1,0) b, (1,3) a a, (3,3) a, (4,3) b, (4,6) a a, (6,6) a, ...
    assert seq == [a, b, a, a, a, b, a, a, a, b, a, a, a, b, a, a]
    assert p.jobs[a].attained == 12 and p.jobs[b].attained == 12
    assert p.jobs[a].served == 12 and p.jobs[b].served == 4
    assert p.set_cost(a, 0) == op.EINVAL and p.set_cost(9, 1) == op.EINVAL


def test_srtf_orders_by_remaining_time():
    p = op.Pool(1 << 20, granule=256, max_lanes=1, policy=op.PRIORITY)
    a = p.job_arrive(4096, 4096, 0, 10)[1]          # 10 iterations of 1   -> 10
    b = p.job_arrive(4096, 4096, 0, 4)[1]           #  4 iterations of 5   -> 20
    c = p.job_arrive(4096, 4096, 0, 6)[1]           #  6 iterations of 2   -> 12
    p.set_cost(b, 5), p.set_cost(c, 2)
    order = []
    while True:
        s = p.schedule_iteration()
        if not s:
            break
        order.append(s[0][0])
    assert order == [a] * 10 + [c] * 6 + [b] * 4    # counting iterations alone would start with b
    # a higher priority still wins over any remaining time
    p = op.Pool(1 << 20, granule=256, max_lanes=1, policy=op.PRIORITY)
    a = p.job_arrive(4096, 4096, 0, 2)[1]
    b = p.job_arrive(4096, 4096, 3, 50)[1]
    p.set_cost(b, 100)
    assert p.schedule_iteration()[0][0] == b
