"""CPU oracle for the memory model, lane assignment and iteration scheduler.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain reference that the
HIP library is compared against.  It shares no code with the product; only
tests, the smoke check and the CPU-baseline leg of the benchmark may import it.

What it follows (Salus, arXiv 1902.04610):

* Section 3.2.1 - persistent (model + framework-internal) versus ephemeral
  memory; persistent memory stays on the GPU for the whole job.
* Section 3.3 - the pool is split into a persistent region and an ephemeral
  region that grow from the two ends; the ephemeral region is cut into lanes.
* Section 3.3.1 - when a lane disappears the lanes behind it take over its
  space at the iteration boundary, without copying anything.
* Algorithm 1 - JobArrive / JobFinish / LaneMoved / ProcessRequests / FindLane.
* Safety condition (Section 3.3.2): sum P_i + sum L_j <= C,  L_j >= max E_i.
* Section 4 - FIFO, SRTF (priority), PACK and FAIR (round-robin) policies, all
  switching jobs only between iterations (Section 3.2.2).

Where the paper is silent the reading taken is written next to the code and
listed in the design document.  Parity status: every function here is pinned
by tests/test_oracle_pool.py (worked examples, invariants, brute force).

Addresses are byte offsets inside a pool of C bytes.  The optional ``mem``
array (numpy uint8, length C) carries the bytes so that switches and
compaction can be checked byte for byte; with ``mem=None`` only metadata is
tracked (used for pools far larger than host memory).
"""

FIFO, RR, PRIORITY, PACK = 0, 1, 2, 3

QUEUED, RESIDENT, EVICTED, DONE = 0, 1, 2, 3

OK, IS_QUEUED = 0, 1
EINVAL, ENOMEM, ENOTRESIDENT, EBUSY, ENEVER = -1, -2, -3, -4, -5

# event kinds, in the order they are appended to Pool.events
EV_ADMIT, EV_EVICT, EV_RESTORE, EV_LANE_NEW, EV_LANE_GROW, EV_LANE_DEL, \
    EV_LANE_MOVED, EV_COMPACT, EV_LANE_SHRINK, EV_LANE_PARK, EV_LANE_UNPARK = range(11)


def round_up(x, a):
    return (x + a - 1) // a * a


class Job:
    def __init__(self, jid, P, E, priority, pending, arrival_round):
        self.id = jid
        self.P = P                  # persistent bytes, granule-rounded
        self.E = E                  # ephemeral peak bytes, granule-rounded
        self.priority = priority    # larger number = more important
        self.pending = pending      # iterations still to run (SRTF: remaining time)
        self.served = 0             # iterations issued so far
        self.cost = 1               # duration of one iteration, in the caller's time unit
        self.attained = 0           # sum of the costs of the iterations issued (FAIR: attained service)
        self.state = QUEUED
        self.lane = -1              # lane id
        self.off = -1               # offset of the persistent block
        self.auto_evicted = False   # evicted by priority admission, restore automatically
        self.host = None            # bytes held on the host while EVICTED
        self.held = False           # persistent bytes in transit: resident but not runnable
        self.arrival_round = arrival_round
        self.admit_round = -1


class Lane:
    def __init__(self, lid, size):
        self.id = lid
        self.size = size            # L_j
        self.ref = 0                # number of jobs assigned (Algorithm 1, ref(lane))


class Pool:
    def __init__(self, capacity, granule=256, max_lanes=0, policy=RR, mem=None, shrink_lanes=False):
        assert capacity > 0 and granule > 0 and capacity % granule == 0
        self.C = capacity
        self.A = granule
        self.max_lanes = max_lanes  # 0 = unlimited
        self.policy = policy
        self.shrink_lanes = shrink_lanes   # keep L_j == max E_i when a lane's largest job leaves
        self.mem = mem
        self.jobs = []              # all jobs ever created, index = job id
        self.lanes = []             # existing lanes in creation order
        self.Q = []                 # pending queue of job ids, arrival order
        self.next_lane_id = 0
        self.round = 0
        self.events = []
        self.stats = dict(rounds=0, iterations=0, bytes_d2h=0, bytes_h2d=0,
                          bytes_d2d=0, moves=0, compactions=0, lanes_opened=0,
                          lanes_deleted=0, lanes_moved=0, evictions=0,
                          restores=0, admitted=0)

    # ---------------------------------------------------------------- layout
    def parked(self, lane, without=()):
        """A lane none of whose jobs is resident (all evicted) reserves no
        memory: nothing can run in it, and ephemeral memory only exists during
        an iteration (Section 3.2.1).  It keeps its id, its jobs and its
        nominal size L_j and takes its bytes back when one of its jobs is
        restored.  Without this, a job admitted by priority (Section 4.2: it
        only has to fit alone) could be blocked for ever by the lanes of the
        jobs evicted for it.  ``without``: jobs to be treated as evicted."""
        return not any(j.state == RESIDENT and j.lane == lane.id and j not in without
                       for j in self.jobs)

    def eff(self, lane, without=()):
        return 0 if self.parked(lane, without) else lane.size

    def sum_L(self, without=()):
        return sum(self.eff(l, without) for l in self.lanes)

    def floor(self):
        """Lowest address of the ephemeral region = end of the persistent region."""
        return self.C - self.sum_L()

    def lane_base(self, lane_id):
        """Lanes stack downward from C in creation order (Section 3.3; which end
        is which is not stated, persistent is taken to be the low end).  The
        base is a closed form of the sizes of the lanes created earlier, so
        deleting a lane moves every later lane up with no bytes copied
        (Section 3.3.1)."""
        top = self.C
        for l in self.lanes:
            top -= self.eff(l)
            if l.id == lane_id:
                return top
        raise KeyError(lane_id)

    def lane_by_id(self, lane_id):
        for l in self.lanes:
            if l.id == lane_id:
                return l
        raise KeyError(lane_id)

    def resident(self):
        return [j for j in self.jobs if j.state == RESIDENT]

    def sum_P(self):
        return sum(j.P for j in self.resident())

    def live_blocks(self):
        """Persistent blocks of resident jobs in ascending address order."""
        return sorted(self.resident(), key=lambda j: j.off)

    def holes(self, floor):
        """Free ranges of the persistent region [0, floor), ascending."""
        out, cur = [], 0
        for j in self.live_blocks():
            if j.off > cur:
                out.append((cur, j.off - cur))
            cur = max(cur, j.off + j.P)
        if floor > cur:
            out.append((cur, floor - cur))
        return out

    def first_fit(self, P, floor):
        for off, size in self.holes(floor):
            if off + P <= floor and size >= P:
                return off
        return None

    # ------------------------------------------------------------ compaction
    def compact(self):
        """Slide every live persistent block to the low end, keeping address
        order.  New offset of the k-th block = sum of the granule-rounded sizes
        of the blocks below it (an exclusive prefix sum).  Blocks that stay
        where they are do not appear in the plan.  The paper only describes
        defragmentation at lane level (Section 3.3.1) and calls the classical
        move-out/move-in scheme costly; how the persistent region itself is
        kept compact is not described, this is the reading taken."""
        plan, new_off = [], 0
        for j in self.live_blocks():
            if j.off != new_off:
                plan.append((j.off, new_off, j.P))
                if self.mem is not None:
                    # memmove semantics: source and destination may overlap
                    self.mem[new_off:new_off + j.P] = self.mem[j.off:j.off + j.P].copy()
                j.off = new_off
            new_off += j.P
        self.stats['compactions'] += 1
        self.stats['moves'] += len(plan)
        self.stats['bytes_d2d'] += sum(m[2] for m in plan)
        self.events.append((EV_COMPACT, len(plan), sum(m[2] for m in plan)))
        return plan

    def place_persistent(self, job, floor):
        """First-fit, lowest address, entirely below ``floor``; compacts first
        when a live block reaches above the floor or no single hole is large
        enough.  The safety condition guarantees that it then fits."""
        high = max((j.off + j.P for j in self.resident()), default=0)
        if high > floor:
            self.compact()
        off = self.first_fit(job.P, floor)
        if off is None:
            self.compact()
            off = self.first_fit(job.P, floor)
        assert off is not None, "safety condition violated"
        job.off = off

    # ------------------------------------------------------- Algorithm 1
    def find_lane(self, P, E, without=()):
        """FindLane of Algorithm 1.  Returns ('new', None) / ('use', lane) /
        ('grow', lane) or None.  ``without`` lists resident jobs to be treated
        as evicted (used to ask "would it fit if these were evicted").

        Readings: the existing-lane branch also needs sum P_i + P + sum L_j <= C
        (the text after the algorithm says a lane is returned only once the
        safety condition is met); "best match" = least slack L_j - E, then
        fewest jobs in the lane, then oldest lane; the replace branch only
        looks at lanes smaller than E (it must never shrink a lane below the
        peak of a job already in it); the number of lanes may be capped; a
        parked lane (no resident job) is invisible here: it holds no memory,
        is not counted, shared or grown."""
        S = sum(j.P for j in self.resident() if j not in without) + P
        lanes = [l for l in self.lanes if not self.parked(l, without)]
        SL = sum(l.size for l in lanes)
        C = self.C
        # open a new lane
        if (self.max_lanes == 0 or len(lanes) < self.max_lanes) and S + SL + E <= C:
            return ('new', None)
        # use an existing lane
        if S + SL <= C:
            fits = [l for l in lanes if l.size >= E]
            if fits:
                return ('use', min(fits, key=lambda l: (l.size - E, l.ref, l.id)))
        # replace (grow) an existing lane, smallest first
        for l in sorted((l for l in lanes if l.size < E), key=lambda l: (l.size, l.id)):
            if S + SL - l.size + E <= C:
                return ('grow', l)
        return None

    def admit(self, job, action):
        kind, lane = action
        if kind == 'new':
            lane = Lane(self.next_lane_id, job.E)
            self.next_lane_id += 1
            new_floor = self.floor() - job.E
        elif kind == 'grow':
            new_floor = self.floor() - (job.E - lane.size)
        else:
            new_floor = self.floor()
        # persistent data above the new floor must move before the lane exists
        high = max((j.off + j.P for j in self.resident()), default=0)
        if high > new_floor:
            self.compact()
        if kind == 'new':
            self.lanes.append(lane)
            self.stats['lanes_opened'] += 1
            self.events.append((EV_LANE_NEW, lane.id, lane.size))
        elif kind == 'grow':
            lane.size = job.E
            self.stats['lanes_moved'] += sum(1 for l in self.lanes if l.id > lane.id)
            self.events.append((EV_LANE_GROW, lane.id, lane.size))
        lane.ref += 1
        job.lane = lane.id
        job.attained = self.lane_service_level(lane.id, job)
        self.place_persistent(job, new_floor)
        job.state = RESIDENT
        job.admit_round = self.round
        self.stats['admitted'] += 1
        self.events.append((EV_ADMIT, job.id, lane.id))

    def lane_service_level(self, lane_id, newcomer):
        """Attained service a job starts with when it enters a lane.  Section 4.3
        equalizes total service over time inside a lane; Section 5.1.2 (fair
        sharing microbenchmark) says that when a further job starts every
        job's share drops to 1/n at once.  A newcomer that started at zero
        would instead receive every iteration until it had caught up with jobs
        that ran before it existed.  Reading taken: service is equalized from
        the moment a job joins, i.e. it starts level with the least-served job
        it competes with - the lane's runnable jobs, or, when none is runnable
        at that moment, the lane's resident jobs; zero in an empty lane."""
        others = [j for j in self.jobs
                  if j is not newcomer and j.state == RESIDENT and j.lane == lane_id]
        runnable = [j for j in others if j.pending > 0 and not j.held]
        level = runnable or others
        return min((j.attained for j in level), default=0)

    def process_requests(self):
        """ProcessRequests of Algorithm 1: every queued request is tried in
        arrival order; one that cannot be placed stays queued and the scan goes
        on (the listing never says that satisfied requests leave Q; they do).

        Under the PRIORITY policy a request that finds no lane may push out
        resident jobs of strictly lower priority (Section 4.2: a higher
        priority job is admitted whenever it could run alone).  The paper never
        moves persistent memory and does not say what happens to the jobs that
        no longer fit; here their persistent state is evicted to host memory,
        lowest priority first, then largest P, then youngest, and only as many
        as needed; nothing is evicted when even evicting all would not help.
        A lane whose jobs are all evicted is parked (see ``parked``), so a
        request whose P + E fits the pool is always admitted when every other
        job has a lower priority."""
        for jid in list(self.Q):
            job = self.jobs[jid]
            action = self.find_lane(job.P, job.E)
            if action is None and self.policy == PRIORITY:
                victims = sorted((v for v in self.resident() if v.priority < job.priority and not v.held),
                                 key=lambda v: (v.priority, -v.P, -v.id))
                need = None
                for n in range(1, len(victims) + 1):
                    if self.find_lane(job.P, job.E, without=victims[:n]) is not None:
                        need = n
                        break
                if need is not None:
                    for v in victims[:need]:
                        self.evict(v, auto=True)
                    action = self.find_lane(job.P, job.E)
            if action is not None:
                self.Q.remove(jid)
                self.admit(job, action)

    def job_arrive(self, P, E, priority=0, pending=0):
        """JobArrive(P, E).  Returns (status, job id)."""
        if P <= 0 or E <= 0:
            return EINVAL, -1
        P, E = round_up(P, self.A), round_up(E, self.A)
        if P + E > self.C:
            return ENEVER, -1       # could not even run alone (Section 4.2)
        job = Job(len(self.jobs), P, E, priority, pending, self.round)
        self.jobs.append(job)
        self.Q.append(job.id)
        self.process_requests()
        return (OK if job.state == RESIDENT else IS_QUEUED), job.id

    def job_finish(self, jid):
        """JobFinish.  The listing re-runs ProcessRequests only when a lane is
        deleted; a finishing job also returns its persistent bytes, which can
        make a queued request feasible, so the queue is processed after every
        finish (otherwise a request could wait for ever with room available)."""
        if not (0 <= jid < len(self.jobs)) or self.jobs[jid].state == DONE:
            return EINVAL
        job = self.jobs[jid]
        if job.held:
            return EBUSY
        if job.state == QUEUED:
            self.Q.remove(jid)
            job.state = DONE
            return OK
        lane = self.lane_by_id(job.lane)
        was_parked = self.parked(lane)
        job.state, job.host = DONE, None
        lane.ref -= 1
        if lane.ref == 0:
            behind = sum(1 for l in self.lanes if l.id > lane.id) if not was_parked else 0
            self.lanes.remove(lane)
            self.stats['lanes_deleted'] += 1
            self.events.append((EV_LANE_DEL, lane.id, 0))
            if behind:
                # auto defragmentation: metadata only, no bytes move
                self.stats['lanes_moved'] += behind
                self.events.append((EV_LANE_MOVED, behind, 0))
        elif self.shrink_lanes:
            # Section 3.3.2 writes L_j = max E_i as an equality, but Algorithm 1
            # never shrinks a lane.  Optional reading: when the job with the
            # largest peak leaves, the lane falls back to the largest remaining
            # peak; ephemeral memory is dead between iterations, so the lanes
            # behind it slide up for free, exactly as after a deletion.
            need = max(j.E for j in self.jobs
                       if j.state in (RESIDENT, EVICTED) and j.lane == lane.id)
            if need < lane.size:
                lane.size = need
                behind = sum(1 for l in self.lanes if l.id > lane.id)
                if not was_parked:
                    self.stats['lanes_moved'] += behind
                self.events.append((EV_LANE_SHRINK, lane.id, need))
        if lane.ref > 0 and not was_parked:
            self.note_parked(lane)
        self.process_requests()
        # bring back jobs that priority admission pushed out, oldest first
        for v in self.jobs:
            if v.state == EVICTED and v.auto_evicted and self.can_restore(v):
                self.switch_in(v.id)
        return OK

    # ------------------------------------------------------------- switching
    def note_parked(self, lane):
        """Called after a job of ``lane`` stopped being resident: if it was the
        last one, the lane is parked from now on and younger lanes slide up."""
        if self.parked(lane):
            self.stats['lanes_moved'] += sum(1 for l in self.lanes if l.id > lane.id)
            self.events.append((EV_LANE_PARK, lane.id, lane.size))

    def can_restore(self, job):
        """Safety condition for bringing an evicted job back; a parked lane
        needs its bytes again, and counts against the lane cap again."""
        lane = self.lane_by_id(job.lane)
        back = 0
        if self.parked(lane):
            active = sum(1 for l in self.lanes if not self.parked(l))
            if self.max_lanes and active >= self.max_lanes:
                return False
            back = lane.size
        return self.sum_P() + job.P + self.sum_L() + back <= self.C

    def evict(self, job, auto):
        if self.mem is not None:
            job.host = self.mem[job.off:job.off + job.P].copy()
        job.state, job.off, job.auto_evicted = EVICTED, -1, auto
        self.stats['evictions'] += 1
        self.stats['bytes_d2h'] += job.P
        self.events.append((EV_EVICT, job.id, job.P))
        self.note_parked(self.lane_by_id(job.lane))

    def switch_out(self, jid):
        if not (0 <= jid < len(self.jobs)):
            return EINVAL
        job = self.jobs[jid]
        if job.state != RESIDENT:
            return ENOTRESIDENT
        if job.held:
            return EBUSY
        self.evict(job, auto=False)
        return OK

    def hold(self, jid):
        """Overlapped switching (the transfer of one job runs while other lanes
        keep iterating, Section 5.1.2 fast job switching): between the start and
        the end of a transfer the job keeps its lane and its persistent block
        but is not runnable, cannot be chosen as an eviction victim and cannot
        finish.  The paper gives no state machine for this; this is the reading
        taken."""
        if not (0 <= jid < len(self.jobs)):
            return EINVAL
        job = self.jobs[jid]
        if job.state != RESIDENT:
            return ENOTRESIDENT
        if job.held:
            return EBUSY
        job.held = True
        return OK

    def release(self, jid):
        if not (0 <= jid < len(self.jobs)) or not self.jobs[jid].held:
            return EINVAL
        self.jobs[jid].held = False
        return OK

    def switch_in(self, jid):
        if not (0 <= jid < len(self.jobs)):
            return EINVAL
        job = self.jobs[jid]
        if job.state != EVICTED:
            return EINVAL
        if not self.can_restore(job):
            return ENOMEM
        lane = self.lane_by_id(job.lane)
        unpark = self.parked(lane)
        # a parked lane takes its bytes back: the block goes below the lowered floor
        self.place_persistent(job, self.floor() - (lane.size if unpark else 0))
        job.state, job.auto_evicted = RESIDENT, False
        if unpark:
            self.stats['lanes_moved'] += sum(1 for l in self.lanes if l.id > lane.id)
            self.events.append((EV_LANE_UNPARK, lane.id, lane.size))
        if self.mem is not None:
            self.mem[job.off:job.off + job.P] = job.host
        job.host = None
        self.stats['restores'] += 1
        self.stats['bytes_h2d'] += job.P
        self.events.append((EV_RESTORE, job.id, job.off))
        return OK

    # ------------------------------------------------------------ scheduling
    def set_pending(self, jid, n):
        if not (0 <= jid < len(self.jobs)) or self.jobs[jid].state == DONE:
            return EINVAL
        self.jobs[jid].pending = n
        return OK

    def set_cost(self, jid, cost):
        """Measured or estimated duration of one iteration of the job (Section 4:
        FAIR equalizes the service *time* jobs have received, SRTF orders by
        remaining *time*).  With the default of 1 for every job both reduce to
        counting iterations."""
        if not (0 <= jid < len(self.jobs)) or self.jobs[jid].state == DONE or cost < 1:
            return EINVAL
        self.jobs[jid].cost = cost
        return OK

    def schedule_iteration(self):
        """One scheduling round: at most one job per lane (iterations are
        serialized inside a lane and run in parallel across lanes, Section
        3.3), chosen among the lane's resident jobs that have an iteration
        pending.  Returns [(job id, lane id)] in lane creation order.

        FAIR/RR  - least attained service (sum of the costs of the iterations
                   issued since the job joined the lane, plus the level it
                   joined at, see lane_service_level); tie: oldest job.
        PRIORITY - highest priority, then shortest remaining time (pending
                   iterations x cost), then oldest (SRTF when priorities are
                   equal; preemption at round boundaries).
        PACK     - every lane runs its oldest runnable job.
        FIFO     - only the oldest runnable job of the whole pool runs."""
        def runnable(lane):
            return [j for j in self.jobs
                    if j.state == RESIDENT and j.lane == lane.id and j.pending > 0 and not j.held]
        picks = []
        if self.policy == FIFO:
            cand = [j for l in self.lanes for j in runnable(l)]
            if cand:
                picks.append(min(cand, key=lambda j: j.id))
        else:
            for lane in self.lanes:
                cand = runnable(lane)
                if not cand:
                    continue
                if self.policy == RR:
                    picks.append(min(cand, key=lambda j: (j.attained, j.id)))
                elif self.policy == PRIORITY:
                    picks.append(min(cand, key=lambda j: (-j.priority, j.pending * j.cost, j.id)))
                else:
                    picks.append(min(cand, key=lambda j: j.id))
        for j in picks:
            j.served += 1
            j.attained += j.cost
            j.pending -= 1
        self.round += 1
        self.stats['rounds'] += 1
        self.stats['iterations'] += len(picks)
        return [(j.id, j.lane) for j in picks]

    # ------------------------------------------------------------ invariants
    def check_invariants(self):
        """Safety condition and layout facts of Section 3.3; raises on violation."""
        A, C = self.A, self.C
        assert self.sum_P() + self.sum_L() <= C
        for l in self.lanes:
            members = [j for j in self.jobs if j.state in (RESIDENT, EVICTED) and j.lane == l.id]
            assert l.ref == len(members) and l.ref > 0
            assert l.size >= max(j.E for j in members)
            if self.shrink_lanes:
                assert l.size == max(j.E for j in members)     # the equality of Section 3.3.2
            assert l.size % A == 0
        # lanes: contiguous, disjoint, stacked below C
        top = C
        for l in self.lanes:
            base = self.lane_base(l.id)
            assert base + self.eff(l) == top
            top = base
        assert top == self.floor()
        if self.max_lanes:
            assert sum(1 for l in self.lanes if not self.parked(l)) <= self.max_lanes
        assert all(j.state == RESIDENT for j in self.jobs if j.held)
        # persistent blocks: disjoint, granule aligned, below the floor
        cur = 0
        for j in self.live_blocks():
            assert j.off % A == 0 and j.off >= cur
            cur = j.off + j.P
        assert cur <= self.floor()
