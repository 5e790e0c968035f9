"""CPU-only checks of the library's host logic.

With a NULL base the pool is metadata-only: allocator, lane assignment,
scheduler, eviction decisions and compaction plans run exactly as on the GPU
but nothing is copied.  Every observable (status codes, offsets, lane bases,
schedules, event log, counters, move plans) must equal the oracle's, bit for bit.
"""
import os
import random
import re

import pytest

from oracle import pool as op
from paper_1902_04610_amd import salus

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "salus.h")).read()
    declared = set(re.findall(r"\b(salus_[a-z0-9_]+)\s*\(", text))
    assert {"salus_pool_create", "salus_lane_alloc", "salus_lane_free", "salus_schedule_iteration",
            "salus_grouped_forward", "salus_switch_out", "salus_switch_in",
            "salus_compact"} <= declared
    L = salus.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert declared == set(salus._PROTOS)        # the binding covers the whole header


def snapshot_oracle(p):
    jobs = []
    for j in p.jobs:
        in_lane = j.state in (op.RESIDENT, op.EVICTED)
        jobs.append((j.state, j.lane if j.state != op.QUEUED else -1, j.P, j.E,
                     j.off if j.state == op.RESIDENT else None,
                     p.lane_base(j.lane) if in_lane else None,
                     p.lane_by_id(j.lane).size if in_lane else 0,
                     j.pending, j.served, int(j.auto_evicted and j.state == op.EVICTED), int(j.held),
                     j.cost, j.attained))
    lanes = [(l.id, p.lane_base(l.id), p.eff(l)) for l in p.lanes]
    return jobs, lanes


def snapshot_lib(p, njobs):
    jobs = []
    for i in range(njobs):
        q = p.job_query(i)
        in_lane = q.state in (salus.JOB_RESIDENT, salus.JOB_EVICTED)
        jobs.append((q.state, q.lane if q.state != salus.JOB_QUEUED else -1, q.P, q.E,
                     q.persist_off if q.state == salus.JOB_RESIDENT else None,
                     q.lane_off if in_lane else None, q.lane_size, q.pending, q.served,
                     int(q.auto_evicted and q.state == salus.JOB_EVICTED), q.in_transit, q.cost, q.attained))
    return jobs, p.lanes()


STAT_KEYS = ("rounds", "iterations", "bytes_d2h", "bytes_h2d", "bytes_d2d", "moves", "compactions",
             "lanes_opened", "lanes_deleted", "lanes_moved", "evictions", "restores", "admitted")


def drive_both(seed, steps, C, granule, max_lanes, policy, size_hi, shrink=False, overlapped=False):
    """overlapped: also split switches into begin / end.  The oracle has no transfers,
    only the rule that a job in transit is held: out_begin = hold, out_end = release +
    switch_out, in_begin = switch_in + hold, in_end = release."""
    rnd = random.Random(seed)
    transit = {}
    o = op.Pool(C, granule=granule, max_lanes=max_lanes, policy=policy, shrink_lanes=shrink)
    g = salus.Pool(None, C, granule=granule, max_lanes=max_lanes, policy=policy,
                   shrink_lanes=shrink)
    for step in range(steps):
        r = rnd.random()
        alive = [j.id for j in o.jobs if j.state != op.DONE]
        if r < 0.40 or not alive:
            P, E = rnd.randint(1, size_hi), rnd.randint(1, size_hi)
            pr, pend = rnd.randint(0, 3), rnd.randint(0, 12)
            so, jo = o.job_arrive(P, E, pr, pend)
            sg, jg = g.lane_alloc(P, E, pr, pend)
            assert (so, jo) == (sg, jg), (seed, step)
        elif r < 0.65:
            jid = rnd.choice(alive + [len(o.jobs) + 3])
            assert o.job_finish(jid) == g.lane_free(jid), (seed, step)
        elif r < 0.85:
            assert o.schedule_iteration() == g.schedule_iteration(), (seed, step)
        elif r < 0.88:
            jid = rnd.choice(alive)
            n = rnd.randint(0, 9)
            assert o.set_pending(jid, n) == g.job_set_pending(jid, n)
        elif r < 0.90:
            jid = rnd.choice(alive + [len(o.jobs) + 1])
            c = rnd.choice([0, 1, 2, 3, 7, 10 ** 12])
            assert o.set_cost(jid, c) == g.job_set_cost(jid, c)
        elif overlapped and r < 0.93:
            jid = rnd.choice(alive + list(transit) * 2)
            if jid in transit:
                if transit.pop(jid) == "out":
                    assert g.switch_out_end(jid, wait=rnd.random() < 0.5) == salus.OK
                    assert o.release(jid) == op.OK and o.switch_out(jid) == op.OK
                else:
                    assert g.switch_in_end(jid) == salus.OK and o.release(jid) == op.OK
            elif o.jobs[jid].state == op.EVICTED:
                rc = o.switch_in(jid)
                assert g.switch_in_begin(jid, None) == rc, (seed, step)
                if rc == op.OK:
                    assert o.hold(jid) == op.OK
                    transit[jid] = "in"
            else:
                rc = o.hold(jid)
                assert g.switch_out_begin(jid, None) == rc, (seed, step)
                if rc == op.OK:
                    transit[jid] = "out"
        elif r < 0.96:
            jid = rnd.choice(alive)
            if o.jobs[jid].state == op.EVICTED:
                assert o.switch_in(jid) == g.switch_in(jid), (seed, step)
            else:
                assert o.switch_out(jid) == g.switch_out(jid), (seed, step)
        else:
            assert o.compact() == g.compact(), (seed, step)
        o.check_invariants()
        assert snapshot_oracle(o) == snapshot_lib(g, len(o.jobs)), (seed, step)
        assert [tuple(e) for e in o.events] == g.poll_events(), (seed, step)
        o.events.clear()
        st = g.stats()
        assert {k: o.stats[k] for k in STAT_KEYS} == {k: st[k] for k in STAT_KEYS}, (seed, step)
        assert st["queued"] == len(o.Q)
    g.close()


@pytest.mark.parametrize("policy", [op.FIFO, op.RR, op.PRIORITY, op.PACK])
def test_random_event_sequences_match_oracle(policy):
    for seed in range(12):
        drive_both(seed * 7 + policy, 250, C=64 * 1024, granule=256,
                   max_lanes=[0, 2, 6][seed % 3], policy=policy, size_hi=12000)


def test_tight_pool_with_many_compactions_matches_oracle():
    for seed in range(8):
        drive_both(100 + seed, 400, C=16 * 1024, granule=16, max_lanes=3, policy=op.RR, size_hi=2500)


@pytest.mark.parametrize("policy", [op.RR, op.PRIORITY, op.PACK])
def test_lane_shrinking_matches_oracle(policy):
    for seed in range(8):
        drive_both(300 + seed * 5 + policy, 300, C=64 * 1024, granule=64,
                   max_lanes=[2, 3, 6][seed % 3], policy=policy, size_hi=9000, shrink=True)


@pytest.mark.parametrize("policy", [op.RR, op.PRIORITY, op.PACK])
def test_overlapped_switching_bookkeeping_matches_oracle(policy):
    for seed in range(10):
        drive_both(500 + seed * 3 + policy, 300, C=64 * 1024, granule=256,
                   max_lanes=[0, 2, 4][seed % 3], policy=policy, size_hi=12000, overlapped=True)


def test_overlapped_switching_error_paths():
    g = salus.Pool(None, 1 << 20)
    st, a = g.lane_alloc(4096, 4096, 0, 3)
    st, b = g.lane_alloc(4096, 4096, 0, 3)
    assert g.switch_out_end(a) == salus.EINVAL                 # nothing begun
    assert g.switch_in_begin(a, None) == salus.EINVAL          # not evicted
    assert g.switch_out_begin(a, None) == salus.OK
    assert g.job_query(a).in_transit == 1 and g.job_query(a).state == salus.JOB_RESIDENT
    assert g.switch_out_begin(a, None) == salus.EBUSY
    assert g.switch_out(a) == salus.EBUSY and g.lane_free(a) == salus.EBUSY
    assert g.switch_in_end(a) == salus.EINVAL                  # wrong direction
    assert [j for j, _ in g.schedule_iteration()] == [b]       # a is not runnable
    assert g.switch_out_end(a) == salus.OK
    assert g.job_query(a).state == salus.JOB_EVICTED and g.job_query(a).in_transit == 0
    assert g.switch_in_begin(a, None) == salus.OK
    assert g.job_query(a).state == salus.JOB_RESIDENT and g.job_query(a).in_transit == 1
    assert [j for j, _ in g.schedule_iteration()] == [b]
    assert g.switch_in_end(a) == salus.OK
    assert sorted(j for j, _ in g.schedule_iteration()) == [a, b]
    g.close()


def test_workload1_layout_through_the_library():
    MiB = 1 << 20
    g = salus.Pool(None, 4 * MiB, granule=256, policy=salus.POLICY_FAIR)
    for _ in range(4):
        assert g.lane_alloc(512 * 1024, MiB, 0, 8)[0] == salus.OK
    rows = [ln.split() for ln in open(os.path.join(ROOT, "tests", "golden", "workload1_layout.txt"))
            if ln.strip() and ln[0] != "#"]
    for job, lane, base, size, off in (map(int, r) for r in rows):
        q = g.job_query(job)
        assert (q.lane, q.lane_off, q.lane_size, q.persist_off) == (lane, base, size, off)
    assert [g.schedule_iteration() for _ in range(4)] == [[(0, 0), (1, 1)], [(2, 0), (3, 1)]] * 2


def test_error_paths_need_no_gpu():
    g = salus.Pool(None, 1 << 20)
    assert g.lane_alloc(1 << 20, 1 << 20)[0] == salus.ENEVER
    assert g.lane_alloc(0, 5)[0] == salus.EINVAL
    st, j = g.lane_alloc(4096, 4096, 0, 1)
    assert st == salus.OK
    assert g.lane_free(99) == salus.EINVAL
    assert g.switch_in(j) == salus.EINVAL             # not evicted
    assert g.switch_out(j) == salus.OK
    assert g.switch_out(j) == salus.ENOTRESIDENT
    assert g.schedule_iteration() == []                # evicted jobs are not runnable
    descs, keep = salus.Pool.make_descs([dict(job=j, M=1, dtype=salus.F32,
                                              layers=[(4, 4, 0, 0)], x_off=0, y_off=256)])
    assert g.grouped_forward(descs) == salus.EINVAL   # no device memory behind this pool
    assert g.lane_free(j) == salus.OK
    assert g.lane_free(j) == salus.EINVAL              # double free
    with pytest.raises(salus.SalusError):
        salus.Pool(None, 1000, granule=48)             # granule must be a power of two


@pytest.mark.parametrize("capacity_gb", [250, 48])
def test_workload5_full_trace_metadata_matches_oracle(capacity_gb):
    """The whole 2000-round fragmentation trace at full sizes, metadata only:
    admissions, queueing, lane churn, compaction plans and byte counters."""
    from paper_1902_04610_amd import synth
    C = capacity_gb * 10 ** 9 // 256 * 256
    trace = synth.workload5_trace(seed=4, rounds=2000)
    o = op.Pool(C, policy=op.RR, max_lanes=6)
    g = salus.Pool(None, C, policy=salus.POLICY_FAIR, max_lanes=6)
    nxt, life = 0, {}
    for rnd in range(2000):
        while nxt < len(trace) and trace[nxt]["arrive"] <= rnd:
            t = trace[nxt]
            so, jo = o.job_arrive(t["P"], t["E"], 0, 10 ** 9)
            assert g.lane_alloc(t["P"], t["E"], 0, 10 ** 9) == (so, jo)
            life[jo] = t["life"]
            nxt += 1
        for j in o.jobs:
            if j.state == op.RESIDENT and rnd - j.admit_round >= life[j.id]:
                assert g.lane_free(j.id) == o.job_finish(j.id) == op.OK
        assert g.schedule_iteration() == o.schedule_iteration()
        if o.events:
            assert [tuple(e) for e in o.events] == g.poll_events(), rnd
            o.events.clear()
            o.check_invariants()
    assert snapshot_oracle(o) == snapshot_lib(g, len(o.jobs))
    st = g.stats()
    assert {k: o.stats[k] for k in STAT_KEYS} == {k: st[k] for k in STAT_KEYS}
    assert len(o.jobs) > 150 and st["lanes_opened"] > 6
    if capacity_gb == 48:
        assert st["compactions"] > 10 and st["bytes_d2d"] > 100 * 10 ** 9
    else:
        assert st["bytes_d2d"] == 0          # the literal pool is never under pressure
    g.close()


def test_workload4_schedule_matches_oracle_over_500_rounds():
    GB = 10 ** 9
    C = 23 * GB // 256 * 256
    o = op.Pool(C, policy=op.PRIORITY)
    g = salus.Pool(None, C, policy=salus.POLICY_PRIORITY)
    assert g.lane_alloc(20 * GB, 2 * GB, 0, 10 ** 9) == o.job_arrive(20 * GB, 2 * GB, 0, 10 ** 9)
    running = None
    for rnd in range(500):
        if rnd and rnd % 50 == 0:
            assert g.lane_alloc(2 * GB, 2 * GB, 5, 10) == o.job_arrive(2 * GB, 2 * GB, 5, 10)
            running = (len(o.jobs) - 1, rnd + 10)
        if running and rnd == running[1]:
            assert g.lane_free(running[0]) == o.job_finish(running[0]) == op.OK
            running = None
        so = o.schedule_iteration()
        assert g.schedule_iteration() == so
        # while the urgent job is resident the evicted job cannot run
        assert [j for j, _ in so] == ([running[0]] if running else [0])
    st = g.stats()
    assert (st["evictions"], st["restores"]) == (9, 9) == (o.stats["evictions"], o.stats["restores"])
    assert st["bytes_d2h"] == st["bytes_h2d"] == 9 * (20 * GB // 256 * 256)
    assert [tuple(e) for e in o.events] == g.poll_events()
    g.close()


def test_priority_job_that_fits_alone_is_admitted_through_the_library():
    """Section 4.2 through the C ABI: the lane of the evicted job is parked, so the
    urgent job (P + E <= C) gets in; the lane and the job come back afterwards."""
    g = salus.Pool(None, 100 * 256, granule=256, policy=salus.POLICY_PRIORITY)
    o = op.Pool(100 * 256, granule=256, policy=op.PRIORITY)
    assert g.lane_alloc(10 * 256, 60 * 256, 0, 50) == o.job_arrive(10 * 256, 60 * 256, 0, 50) == (salus.OK, 0)
    assert g.lane_alloc(50 * 256, 45 * 256, 9, 5) == o.job_arrive(50 * 256, 45 * 256, 9, 5) == (salus.OK, 1)
    low, high = g.job_query(0), g.job_query(1)
    assert low.state == salus.JOB_EVICTED and low.lane_parked == 1 and low.lane_size == 60 * 256
    assert high.lane_parked == 0 and high.lane_off == 55 * 256 and high.persist_off == 0
    assert g.lanes() == [(0, 100 * 256, 0), (1, 55 * 256, 45 * 256)]
    assert g.schedule_iteration() == o.schedule_iteration() == [(1, 1)]
    assert g.switch_in(0) == o.switch_in(0) == salus.ENOMEM
    assert g.lane_free(1) == o.job_finish(1) == salus.OK
    low = g.job_query(0)
    assert low.state == salus.JOB_RESIDENT and low.lane_parked == 0 and low.lane_off == 40 * 256
    assert [tuple(e) for e in o.events] == g.poll_events()
    g.close()


def test_pack_strip128_is_the_documented_permutation():
    import numpy as np
    rng = np.random.default_rng(0)
    for K, N in [(8, 128), (40, 384), (1024, 1024)]:
        w = rng.integers(0, 1 << 16, (K, N), dtype=np.uint16)
        got = salus.pack_strip128(w)
        # element (k, n) sits at (n // 128 * K + k) * 128 + n % 128
        k, n = np.meshgrid(np.arange(K), np.arange(N), indexing="ij")
        want = np.empty(K * N, np.uint16)
        want[(n // 128 * K + k) * 128 + n % 128] = w
        assert np.array_equal(got, want)
    with pytest.raises(salus.SalusError):
        salus.pack_strip128(np.zeros((8, 64), np.uint16))          # N must be a multiple of 128
