"""Trace replay (Section 5.1.1): the library's admission + scheduling against the
oracle's on a whole 100-job trace, hand-worked small traces, and the relations
between policies that the paper states in prose."""
import pytest

from oracle import pool as op
from paper_1902_04610_amd import replay, synth

CAP = 16 * 10 ** 9 // 256 * 256


class OraclePool:
    """The oracle behind the four calls the replay needs."""

    def __init__(self, policy, capacity):
        kind = {"FIFO": op.FIFO, "SRTF": op.PRIORITY, "PACK": op.PACK, "FAIR": op.RR}[policy]
        self.p = op.Pool(capacity, policy=kind, max_lanes=0 if policy == "PACK" else 1)

    def lane_alloc(self, P, E, priority, pending):
        st, jid = self.p.job_arrive(P, E, priority, pending)
        return (1 if st == op.IS_QUEUED else st), jid

    def job_set_cost(self, jid, cost):
        return self.p.set_cost(jid, cost)

    def schedule_iteration(self):
        return self.p.schedule_iteration()

    def lane_free(self, jid):
        return self.p.job_finish(jid)


def job(arrival, iters, cost, util=500, P=4096, E=4096):
    return dict(arrival=arrival, P=P, E=E, iters=iters, cost=cost, util=util)


def run(policy, trace, capacity=CAP, oracle=False):
    pool = OraclePool(policy, capacity) if oracle else replay.library_pool(policy, capacity)
    return replay.replay(pool, trace)


@pytest.mark.parametrize("oracle", [False, True])
def test_hand_worked_three_jobs(oracle):
    trace = [job(0, 3, 10), job(5, 1, 4), job(5, 2, 3)]
    # FIFO: A keeps the GPU until 30, then B (4), then C (3 + 3)
    assert run("FIFO", trace, oracle=oracle) == dict(
        jobs=[(0, 0, 0, 30), (1, 5, 30, 34), (2, 5, 34, 40)], makespan=40)
    # SRTF: at t = 10 the remaining times are A 20, B 4, C 6
    assert run("SRTF", trace, oracle=oracle) == dict(
        jobs=[(0, 0, 0, 40), (1, 5, 10, 14), (2, 5, 14, 20)], makespan=40)


@pytest.mark.parametrize("oracle", [False, True])
def test_packed_round_lasts_as_long_as_the_combined_demand(oracle):
    trace = [job(0, 2, 10, util=800), job(0, 1, 10, util=500)]
    # both lanes run: max(10, 8 + 5) = 13; then A alone: 10
    assert run("PACK", trace, oracle=oracle) == dict(jobs=[(0, 0, 0, 23), (1, 0, 0, 13)], makespan=23)
    # time-shared instead: 10 + 10 + 10
    assert run("FIFO", trace, oracle=oracle)["makespan"] == 30


@pytest.mark.parametrize("policy", replay.POLICIES)
def test_library_and_oracle_replay_the_trace_identically(policy):
    trace = synth.workload_trace100(seed=6)
    assert run(policy, trace) == run(policy, trace, oracle=True)


def test_policy_relations_stated_in_the_paper():
    trace = synth.workload_trace100(seed=6)
    s = {p: replay.summary(run(p, trace)) for p in replay.POLICIES}
    # time sharing adds no overhead: FIFO, SRTF and FAIR finish together; packing is not slower
    assert s["SRTF"]["makespan"] == s["FIFO"]["makespan"] == s["FAIR"]["makespan"]
    assert s["PACK"]["makespan"] <= s["FIFO"]["makespan"]
    # known durations: SRTF cuts the average JCT severalfold; FAIR lies between
    assert s["SRTF"]["avg_jct"] * 2 < s["FIFO"]["avg_jct"]
    assert s["SRTF"]["avg_jct"] < s["FAIR"]["avg_jct"] < s["FIFO"]["avg_jct"]
    assert s["SRTF"]["avg_queuing"] < s["FIFO"]["avg_queuing"]
    assert s["FAIR"]["avg_queuing"] < s["FIFO"]["avg_queuing"]
    # when the jobs arrive together packing shortens the makespan clearly (Section 5.2)
    burst = [dict(j, arrival=0) for j in trace[:24]]
    together = {p: run(p, burst, capacity=4 * CAP)["makespan"] for p in ("FIFO", "PACK")}
    assert together["PACK"] < 0.8 * together["FIFO"]
