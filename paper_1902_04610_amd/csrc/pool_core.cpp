// Host logic of the pool.  See pool_core.hpp for the map to the paper.
#include "pool_core.hpp"

#include <algorithm>

namespace salus {

static inline uint64_t round_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

PoolCore::PoolCore(uint64_t capacity, uint64_t granule, uint32_t max_lanes, int32_t policy,
                   bool shrink_lanes, DeviceOps *dev)
    : C_(capacity), A_(granule), max_lanes_(max_lanes), policy_(policy),
      shrink_lanes_(shrink_lanes), dev_(dev) {}

PoolCore::~PoolCore()
{
    for (Job &j : jobs_)
        if (j.host && j.host_owned) dev_->pinned_free(j.host);
}

// Section 3.3: lanes are stacked downward from the top of the pool in creation
// order, so a lane's base is a running sum over the lanes created before it and
// a deleted lane's space is taken over by its younger neighbours without any
// copy (Section 3.3.1).
uint64_t PoolCore::lane_base(int32_t lane_id, uint64_t *size) const
{
    uint64_t top = C_;
    for (const Lane &l : lanes_) {
        top -= l.bytes();
        if (l.id == lane_id) {
            if (size) *size = l.bytes();
            return top;
        }
    }
    if (size) *size = 0;
    return UINT64_MAX;
}

size_t PoolCore::lane_index(int32_t lane_id) const
{
    for (size_t i = 0; i < lanes_.size(); ++i)
        if (lanes_[i].id == lane_id) return i;
    return lanes_.size();
}

// FindLane of Algorithm 1 under the safety condition of Section 3.3.2.
// residentP = persistent bytes of the jobs that would stay resident.  Parked
// lanes are invisible: they hold no bytes and are not counted, shared or grown.
PoolCore::Choice PoolCore::find_lane(uint64_t P, uint64_t E, uint64_t residentP,
                                     const std::vector<uint32_t> *gone) const
{
    const uint64_t S = residentP + P;
    auto active = [&](size_t i) { return lanes_[i].resident > (gone ? (*gone)[i] : 0u); };
    uint64_t SL = 0;
    size_t count = 0;
    for (size_t i = 0; i < lanes_.size(); ++i)
        if (active(i)) { SL += lanes_[i].size; ++count; }
    Choice c;
    // 1. open a new lane
    if ((max_lanes_ == 0 || count < max_lanes_) && S + SL + E <= C_) {
        c.kind = NEW;
        return c;
    }
    // 2. share an existing lane that is large enough: least slack, then fewest
    //    jobs, then oldest
    if (S + SL <= C_) {
        bool found = false;
        for (size_t i = 0; i < lanes_.size(); ++i) {
            const Lane &l = lanes_[i];
            if (!active(i) || l.size < E) continue;
            if (!found) { found = true; c.index = i; continue; }
            const Lane &b = lanes_[c.index];
            if (l.size - E < b.size - E || (l.size == b.size && l.ref < b.ref)) c.index = i;
        }
        if (found) { c.kind = USE; return c; }
    }
    // 3. grow a lane that is too small, smallest first (oldest among equals)
    std::vector<size_t> small;
    for (size_t i = 0; i < lanes_.size(); ++i)
        if (active(i) && lanes_[i].size < E) small.push_back(i);
    std::stable_sort(small.begin(), small.end(),
                     [&](size_t a, size_t b) { return lanes_[a].size < lanes_[b].size; });
    for (size_t i : small)
        if (S + SL - lanes_[i].size + E <= C_) {
            c.kind = GROW;
            c.index = i;
            return c;
        }
    return c;
}

bool PoolCore::first_fit(uint64_t P, uint64_t fl, uint64_t *off) const
{
    uint64_t cur = 0;
    for (const auto &kv : blocks_) {
        if (kv.first >= cur + P && cur + P <= fl) { *off = cur; return true; }
        cur = kv.first + jobs_[kv.second].P;
    }
    if (fl >= cur && fl - cur >= P) { *off = cur; return true; }
    return false;
}

int PoolCore::do_compact(std::vector<salus_move> *plan_out)
{
    // New offset of each live block = exclusive prefix sum of the sizes below it.
    std::vector<salus_move> plan;
    std::map<uint64_t, int32_t> packed;
    uint64_t next = 0, bytes = 0;
    for (const auto &kv : blocks_) {
        Job &j = jobs_[kv.second];
        if (kv.first != next) {
            plan.push_back({kv.first, next, j.P});
            bytes += j.P;
        }
        packed.emplace_hint(packed.end(), next, kv.second);
        next += j.P;
    }
    int rc = 0;
    if (!plan.empty() && dev_->present()) rc = dev_->slide(plan.data(), (uint32_t)plan.size());
    if (rc) { error = "device compaction failed"; return SALUS_EHIP; }
    for (const auto &kv : packed) jobs_[kv.second].off = kv.first;
    blocks_.swap(packed);
    stats.compactions += 1;
    stats.moves += plan.size();
    stats.bytes_d2d += bytes;
    log(SALUS_EV_COMPACT, plan.size(), bytes);
    if (plan_out) plan_out->swap(plan);
    return SALUS_OK;
}

int32_t PoolCore::compact(std::vector<salus_move> *plan) { return do_compact(plan); }

int PoolCore::place(Job &j, uint64_t fl)
{
    uint64_t high = blocks_.empty() ? 0 : blocks_.rbegin()->first + jobs_[blocks_.rbegin()->second].P;
    if (high > fl)
        if (int rc = do_compact(nullptr)) return rc;
    uint64_t off;
    if (!first_fit(j.P, fl, &off)) {
        if (int rc = do_compact(nullptr)) return rc;
        if (!first_fit(j.P, fl, &off)) { error = "internal: safety condition violated"; return SALUS_ENOMEM; }
    }
    j.off = off;
    blocks_[off] = j.id;
    return SALUS_OK;
}

int PoolCore::admit(Job &j, Choice c)
{
    uint64_t new_floor = floor();
    if (c.kind == NEW) new_floor -= j.E;
    else if (c.kind == GROW) new_floor -= j.E - lanes_[c.index].size;
    // persistent blocks in the way of the lane move down before the lane exists
    uint64_t high = blocks_.empty() ? 0 : blocks_.rbegin()->first + jobs_[blocks_.rbegin()->second].P;
    if (high > new_floor)
        if (int rc = do_compact(nullptr)) return rc;
    const uint64_t old_size = c.kind == GROW ? lanes_[c.index].size : 0;
    const uint64_t old_moved = stats.lanes_moved;
    const size_t mark = events.size();
    if (c.kind == NEW) {
        lanes_.push_back({next_lane_, j.E, 0, 0});
        c.index = lanes_.size() - 1;
        sumL_ += j.E;
        log(SALUS_EV_LANE_NEW, next_lane_, j.E);
    } else if (c.kind == GROW) {
        Lane &l = lanes_[c.index];
        sumL_ += j.E - l.size;
        l.size = j.E;
        stats.lanes_moved += lanes_.size() - 1 - c.index;
        log(SALUS_EV_LANE_GROW, l.id, l.size);
    }
    if (int rc = place(j, floor())) {
        // the device failed while making room: the lane change is undone and
        // the request stays where it was
        if (c.kind == NEW) {
            sumL_ -= j.E;
            lanes_.pop_back();
        } else if (c.kind == GROW) {
            sumL_ -= j.E - old_size;
            lanes_[c.index].size = old_size;
            stats.lanes_moved = old_moved;
        }
        if (c.kind != USE) events.erase(events.begin() + mark);
        return rc;
    }
    Lane &l = lanes_[c.index];
    if (c.kind == NEW) {
        next_lane_ += 1;
        stats.lanes_opened += 1;
    }
    l.ref += 1;
    l.resident += 1;
    j.lane = l.id;
    j.attained = entry_level(j);
    j.state = SALUS_JOB_RESIDENT;
    sumP_ += j.P;
    j.admit_round = round_;
    stats.admitted += 1;
    log(SALUS_EV_ADMIT, j.id, l.id);
    return SALUS_OK;
}

// FAIR (Section 4.3) equalizes service inside a lane; the fair-sharing run of
// Section 5.1.2 shows every job's share dropping to 1/n as soon as a further job
// starts.  A job therefore enters its lane level with the least-served job it
// competes with (runnable jobs first, else resident ones), not at zero: starting
// at zero would hand it every iteration until it had caught up.
uint64_t PoolCore::entry_level(const Job &j) const
{
    uint64_t lo[2] = {UINT64_MAX, UINT64_MAX};      // [0] runnable, [1] resident
    for (const Job &o : jobs_) {
        if (o.id == j.id || o.state != SALUS_JOB_RESIDENT || o.lane != j.lane) continue;
        lo[1] = std::min(lo[1], o.attained);
        if (o.pending > 0 && !o.held) lo[0] = std::min(lo[0], o.attained);
    }
    return lo[0] != UINT64_MAX ? lo[0] : lo[1] != UINT64_MAX ? lo[1] : 0;
}

int PoolCore::host_buffer(Job &j, void *pinned)
{
    if (pinned) {
        if (j.host && j.host_owned) dev_->pinned_free(j.host);
        j.host = pinned;
        j.host_owned = false;
    } else if (!j.host || !j.host_owned) {
        j.host = dev_->pinned_alloc(j.P);
        j.host_owned = true;
        if (!j.host) { error = "pinned host allocation failed"; return SALUS_EHIP; }
    }
    return SALUS_OK;
}

int PoolCore::evict(Job &j, bool automatic, void *pinned, bool copied)
{
    if (dev_->present() && !copied) {
        if (int rc = host_buffer(j, pinned)) return rc;
        if (dev_->evict(j.host, j.off, j.P)) { error = "device-to-host copy failed"; return SALUS_EHIP; }
    }
    blocks_.erase(j.off);
    sumP_ -= j.P;
    j.state = SALUS_JOB_EVICTED;
    j.auto_evicted = automatic;
    stats.evictions += 1;
    stats.bytes_d2h += j.P;
    log(SALUS_EV_EVICT, j.id, j.P);
    left_device(j);
    return SALUS_OK;
}

// One resident job fewer in j's lane; with none left the lane is parked and the
// younger lanes slide up (bookkeeping only).
void PoolCore::left_device(Job &j)
{
    const size_t i = lane_index(j.lane);
    Lane &l = lanes_[i];
    if (--l.resident == 0 && l.ref > 0) {
        sumL_ -= l.size;
        stats.lanes_moved += lanes_.size() - 1 - i;
        log(SALUS_EV_LANE_PARK, l.id, l.size);
    }
}

// Safety condition for bringing an evicted job back: a parked lane needs its
// bytes again and counts against the lane cap again.
bool PoolCore::can_restore(const Job &j) const
{
    const Lane &l = lanes_[lane_index(j.lane)];
    uint64_t back = 0;
    if (l.parked()) {
        size_t active = 0;
        for (const Lane &o : lanes_) active += !o.parked();
        if (max_lanes_ && active >= max_lanes_) return false;
        back = l.size;
    }
    return sumP_ + j.P + sumL_ + back <= C_;
}

// ProcessRequests of Algorithm 1, plus priority admission (Section 4.2).
void PoolCore::process_requests()
{
    std::vector<int32_t> waiting(queue_.begin(), queue_.end());
    for (int32_t id : waiting) {
        Job &j = jobs_[id];
        Choice c = find_lane(j.P, j.E, sumP_);
        if (c.kind == NONE && policy_ == SALUS_POLICY_PRIORITY) {
            // candidates: strictly lower priority; lowest priority first, then
            // largest persistent state, then youngest
            std::vector<int32_t> victims;
            for (const Job &v : jobs_)
                if (v.state == SALUS_JOB_RESIDENT && v.priority < j.priority && !v.held)
                    victims.push_back(v.id);
            std::sort(victims.begin(), victims.end(), [&](int32_t a, int32_t b) {
                const Job &x = jobs_[a], &y = jobs_[b];
                if (x.priority != y.priority) return x.priority < y.priority;
                if (x.P != y.P) return x.P > y.P;
                return x.id > y.id;
            });
            uint64_t left = sumP_;
            size_t need = 0;
            std::vector<uint32_t> gone(lanes_.size(), 0);
            for (size_t n = 0; n < victims.size(); ++n) {
                left -= jobs_[victims[n]].P;
                gone[lane_index(jobs_[victims[n]].lane)] += 1;
                if (find_lane(j.P, j.E, left, &gone).kind != NONE) { need = n + 1; break; }
            }
            for (size_t n = 0; n < need; ++n)
                if (evict(jobs_[victims[n]], true, nullptr)) return;
            if (need) c = find_lane(j.P, j.E, sumP_);
        }
        if (c.kind != NONE) {
            if (admit(j, c)) return;        // the request stays queued when the device fails
            queue_.erase(std::find(queue_.begin(), queue_.end(), id));
        }
    }
}

int32_t PoolCore::arrive(uint64_t P, uint64_t E, int32_t priority, uint64_t pending, int32_t *job)
{
    if (job) *job = -1;
    if (P == 0 || E == 0) { error = "P and E must be positive"; return SALUS_EINVAL; }
    P = round_up(P, A_);
    E = round_up(E, A_);
    if (P + E > C_ || P + E < P) { error = "P + E exceeds the pool capacity"; return SALUS_ENEVER; }
    Job j;
    j.id = (int32_t)jobs_.size();
    j.P = P;
    j.E = E;
    j.priority = priority;
    j.pending = pending;
    j.arrival_round = round_;
    jobs_.push_back(j);
    queue_.push_back(j.id);
    error.clear();
    process_requests();
    if (job) *job = j.id;
    if (!error.empty()) return SALUS_EHIP;
    return jobs_[j.id].state == SALUS_JOB_RESIDENT ? SALUS_OK : SALUS_QUEUED;
}

int32_t PoolCore::finish(int32_t id)
{
    if (id < 0 || (size_t)id >= jobs_.size() || jobs_[id].state == SALUS_JOB_DONE) {
        error = "no such live job";
        return SALUS_EINVAL;
    }
    Job &j = jobs_[id];
    if (j.held) { error = "job is in transit"; return SALUS_EBUSY; }
    if (j.state == SALUS_JOB_QUEUED) {
        queue_.erase(std::find(queue_.begin(), queue_.end(), id));
        j.state = SALUS_JOB_DONE;
        return SALUS_OK;
    }
    const bool was_resident = j.state == SALUS_JOB_RESIDENT;
    if (was_resident) {
        blocks_.erase(j.off);
        sumP_ -= j.P;
    }
    if (j.host && j.host_owned) dev_->pinned_free(j.host);
    j.host = nullptr;
    j.state = SALUS_JOB_DONE;
    const size_t i = lane_index(j.lane);
    const bool was_parked = lanes_[i].parked();
    if (--lanes_[i].ref == 0) {
        const uint64_t behind = was_parked ? 0 : lanes_.size() - 1 - i;
        sumL_ -= lanes_[i].bytes();
        log(SALUS_EV_LANE_DEL, lanes_[i].id, 0);
        lanes_.erase(lanes_.begin() + i);
        stats.lanes_deleted += 1;
        if (behind) {   // younger lanes slide: bookkeeping only
            stats.lanes_moved += behind;
            log(SALUS_EV_LANE_MOVED, behind, 0);
        }
    } else {
        if (shrink_lanes_) {
            // Section 3.3.2 states L_j = max E_i; fall back to the largest peak
            // still in the lane (younger lanes slide up, nothing is copied)
            uint64_t need = 0;
            for (const Job &m : jobs_)
                if ((m.state == SALUS_JOB_RESIDENT || m.state == SALUS_JOB_EVICTED) &&
                    m.lane == lanes_[i].id)
                    need = std::max(need, m.E);
            if (need < lanes_[i].size) {
                if (!was_parked) {
                    sumL_ -= lanes_[i].size - need;
                    stats.lanes_moved += lanes_.size() - 1 - i;
                }
                lanes_[i].size = need;
                log(SALUS_EV_LANE_SHRINK, lanes_[i].id, need);
            }
        }
        if (was_resident) left_device(j);     // may park the lane: only evicted jobs remain
    }
    error.clear();
    process_requests();
    for (size_t v = 0; v < jobs_.size(); ++v)
        if (jobs_[v].state == SALUS_JOB_EVICTED && jobs_[v].auto_evicted && can_restore(jobs_[v]))
            if (switch_in((int32_t)v)) break;
    return error.empty() ? SALUS_OK : SALUS_EHIP;
}

int32_t PoolCore::switch_out(int32_t id, void *pinned)
{
    if (id < 0 || (size_t)id >= jobs_.size()) { error = "no such job"; return SALUS_EINVAL; }
    if (jobs_[id].state != SALUS_JOB_RESIDENT) { error = "job is not resident"; return SALUS_ENOTRESIDENT; }
    if (jobs_[id].held) { error = "job is in transit"; return SALUS_EBUSY; }
    return evict(jobs_[id], false, pinned);
}

int32_t PoolCore::begin_out(int32_t id, void *pinned, void **host, uint64_t *off, uint64_t *len)
{
    if (id < 0 || (size_t)id >= jobs_.size()) { error = "no such job"; return SALUS_EINVAL; }
    Job &j = jobs_[id];
    if (j.state != SALUS_JOB_RESIDENT) { error = "job is not resident"; return SALUS_ENOTRESIDENT; }
    if (j.held) { error = "job is in transit"; return SALUS_EBUSY; }
    if (dev_->present())
        if (int rc = host_buffer(j, pinned)) return rc;
    j.held = j.leaving = true;
    *host = j.host;
    *off = j.off;
    *len = j.P;
    return SALUS_OK;
}

int32_t PoolCore::end_out(int32_t id)
{
    if (id < 0 || (size_t)id >= jobs_.size() || !jobs_[id].held || !jobs_[id].leaving) {
        error = "no device-to-host transfer was begun for this job";
        return SALUS_EINVAL;
    }
    Job &j = jobs_[id];
    j.held = j.leaving = false;
    return evict(j, false, nullptr, true);
}

int32_t PoolCore::begin_in(int32_t id, void **host, uint64_t *off, uint64_t *len)
{
    if (int32_t rc = switch_in_impl(id, false)) return rc;
    Job &j = jobs_[id];
    j.held = true;
    j.leaving = false;
    *host = j.host;
    *off = j.off;
    *len = j.P;
    return SALUS_OK;
}

int32_t PoolCore::end_in(int32_t id)
{
    if (id < 0 || (size_t)id >= jobs_.size() || !jobs_[id].held || jobs_[id].leaving) {
        error = "no host-to-device transfer was begun for this job";
        return SALUS_EINVAL;
    }
    Job &j = jobs_[id];
    j.held = false;
    if (!j.host_owned) j.host = nullptr;
    return SALUS_OK;
}

void PoolCore::drop_hold(int32_t id)
{
    if (id >= 0 && (size_t)id < jobs_.size()) jobs_[id].held = jobs_[id].leaving = false;
}

int32_t PoolCore::switch_in(int32_t id) { return switch_in_impl(id, true); }

int32_t PoolCore::switch_in_impl(int32_t id, bool copy_now)
{
    if (id < 0 || (size_t)id >= jobs_.size() || jobs_[id].state != SALUS_JOB_EVICTED) {
        error = "job is not evicted";
        return SALUS_EINVAL;
    }
    Job &j = jobs_[id];
    if (!can_restore(j)) { error = "no room to restore the job"; return SALUS_ENOMEM; }
    const size_t li = lane_index(j.lane);
    Lane &l = lanes_[li];
    const bool unpark = l.parked();
    // a parked lane takes its bytes back: the block goes below the lowered floor
    // (blocks in the way are compacted while the old floor still holds)
    if (int rc = place(j, floor() - (unpark ? l.size : 0))) return rc;
    if (unpark) {
        sumL_ += l.size;
        stats.lanes_moved += lanes_.size() - 1 - li;
        log(SALUS_EV_LANE_UNPARK, l.id, l.size);
    }
    l.resident += 1;
    j.state = SALUS_JOB_RESIDENT;
    j.auto_evicted = false;
    sumP_ += j.P;
    if (copy_now) {
        if (dev_->present() && dev_->restore(j.off, j.host, j.P)) {
            error = "host-to-device copy failed";
            return SALUS_EHIP;
        }
        if (!j.host_owned) j.host = nullptr;    // the caller's buffer is released; ours stays cached
    }
    stats.restores += 1;
    stats.bytes_h2d += j.P;
    log(SALUS_EV_RESTORE, j.id, j.off);
    return SALUS_OK;
}

int32_t PoolCore::set_pending(int32_t id, uint64_t n)
{
    if (id < 0 || (size_t)id >= jobs_.size() || jobs_[id].state == SALUS_JOB_DONE) {
        error = "no such live job";
        return SALUS_EINVAL;
    }
    jobs_[id].pending = n;
    return SALUS_OK;
}

int32_t PoolCore::set_cost(int32_t id, uint64_t cost)
{
    if (id < 0 || (size_t)id >= jobs_.size() || jobs_[id].state == SALUS_JOB_DONE || cost < 1) {
        error = "no such live job, or a cost of zero";
        return SALUS_EINVAL;
    }
    jobs_[id].cost = cost;
    return SALUS_OK;
}

int32_t PoolCore::query(int32_t id, salus_job_info *o) const
{
    if (id < 0 || (size_t)id >= jobs_.size() || !o) return SALUS_EINVAL;
    const Job &j = jobs_[id];
    o->state = j.state;
    o->lane = j.lane;
    o->priority = j.priority;
    o->auto_evicted = j.auto_evicted;
    o->in_transit = j.held;
    o->lane_parked = 0;
    o->P = j.P;
    o->E = j.E;
    o->persist_off = j.state == SALUS_JOB_RESIDENT ? j.off : UINT64_MAX;
    o->lane_off = UINT64_MAX;
    o->lane_size = 0;
    if (j.state == SALUS_JOB_RESIDENT || j.state == SALUS_JOB_EVICTED) {
        const Lane &l = lanes_[lane_index(j.lane)];
        o->lane_off = lane_base(j.lane);
        o->lane_size = l.size;
        o->lane_parked = l.parked();
    }
    o->pending = j.pending;
    o->served = j.served;
    o->cost = j.cost;
    o->attained = j.attained;
    o->arrival_round = j.arrival_round;
    o->admit_round = j.admit_round;
    return SALUS_OK;
}

// One round: at most one job per lane (iterations are serialized within a lane
// and parallel across lanes, Section 3.3), switching only between iterations
// (Section 3.2.2), under the policies of Section 4.
int32_t PoolCore::schedule(salus_slot *out, uint32_t cap, uint32_t *n)
{
    if (!n || (!out && cap)) return SALUS_EINVAL;
    if (cap < lanes_.size()) { error = "slot array smaller than the number of lanes"; return SALUS_EINVAL; }
    // best runnable job per lane id in one pass over the jobs
    std::map<int32_t, int32_t> best;    // lane id -> job id
    auto better = [&](const Job &a, const Job &b) {
        switch (policy_) {
        case SALUS_POLICY_FAIR:
            return a.attained != b.attained ? a.attained < b.attained : a.id < b.id;
        case SALUS_POLICY_PRIORITY: {
            if (a.priority != b.priority) return a.priority > b.priority;
            // remaining time; 128-bit so that pending = 10^9 with large costs cannot wrap
            const unsigned __int128 ra = (unsigned __int128)a.pending * a.cost,
                                    rb = (unsigned __int128)b.pending * b.cost;
            if (ra != rb) return ra < rb;
            return a.id < b.id;
        }
        default:
            return a.id < b.id;
        }
    };
    for (const Job &j : jobs_) {
        if (j.state != SALUS_JOB_RESIDENT || j.pending == 0 || j.held) continue;
        auto it = best.find(j.lane);
        if (it == best.end()) best[j.lane] = j.id;
        else if (better(j, jobs_[it->second])) it->second = j.id;
    }
    uint32_t k = 0;
    if (policy_ == SALUS_POLICY_FIFO) {
        int32_t pick = -1;
        for (const auto &kv : best)
            if (pick < 0 || kv.second < pick) pick = kv.second;
        if (pick >= 0) out[k++] = {pick, jobs_[pick].lane};
    } else {
        for (const Lane &l : lanes_) {
            auto it = best.find(l.id);
            if (it != best.end()) out[k++] = {it->second, l.id};
        }
    }
    for (uint32_t i = 0; i < k; ++i) {
        jobs_[out[i].job].served += 1;
        jobs_[out[i].job].attained += jobs_[out[i].job].cost;
        jobs_[out[i].job].pending -= 1;
    }
    *n = k;
    round_ += 1;
    stats.rounds += 1;
    stats.iterations += k;
    return SALUS_OK;
}

}  // namespace salus
