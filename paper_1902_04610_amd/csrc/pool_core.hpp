// Host side of the pool: persistent-region allocator, lane assignment
// (Algorithm 1 of the Salus paper), safety condition (Section 3.3.2),
// iteration scheduler (Section 4) and the planners for switching and
// compaction.  Pure C++, no GPU calls: data movement goes through DeviceOps.
#pragma once
#include <cstdint>
#include <deque>
#include <map>
#include <string>
#include <vector>

#include "salus.h"

namespace salus {

// What the host logic needs from the device side.  Offsets are relative to the
// pool base.  Every call is complete (synchronised) when it returns 0.
struct DeviceOps {
    virtual ~DeviceOps() {}
    virtual bool present() const = 0;                       // false: metadata-only pool
    virtual int evict(void *host, uint64_t off, uint64_t n) = 0;      // device -> host
    virtual int restore(uint64_t off, const void *host, uint64_t n) = 0;
    // moves in ascending address order, every dst below its src, a move may overlap
    // its own destination; nothing outside the moved ranges may be touched (lanes
    // hold inputs and outputs that callers keep across rounds, and other lanes may
    // be iterating while a switch_in compacts)
    virtual int slide(const salus_move *moves, uint32_t n) = 0;
    virtual void *pinned_alloc(uint64_t n) = 0;
    virtual void pinned_free(void *p) = 0;
};

struct Job {
    int32_t id = -1;
    uint64_t P = 0, E = 0;
    int32_t priority = 0;
    uint64_t pending = 0, served = 0;
    uint64_t cost = 1, attained = 0;   // iteration duration (caller's unit), sum of issued costs
    int32_t state = SALUS_JOB_QUEUED;
    int32_t lane = -1;
    uint64_t off = 0;
    bool auto_evicted = false;
    void *host = nullptr;        // evicted bytes, or a cached pinned buffer
    bool host_owned = false;     // allocated by the library
    bool held = false;           // persistent bytes in transit: resident, not runnable
    bool leaving = false;        // held by begin_out (the transfer is device -> host)
    uint64_t arrival_round = 0, admit_round = UINT64_MAX;
};

struct Lane {
    int32_t id;
    uint64_t size;               // L_j
    uint32_t ref;                // jobs assigned to the lane
    uint32_t resident;           // of those, jobs whose persistent state is on the device
    // A lane without a resident job is parked: nothing can run in it, so it
    // reserves no bytes until one of its jobs is restored (it keeps id, jobs and L_j).
    bool parked() const { return resident == 0; }
    uint64_t bytes() const { return resident ? size : 0; }
};

class PoolCore {
public:
    PoolCore(uint64_t capacity, uint64_t granule, uint32_t max_lanes, int32_t policy,
             bool shrink_lanes, DeviceOps *dev);
    ~PoolCore();

    int32_t arrive(uint64_t P, uint64_t E, int32_t priority, uint64_t pending, int32_t *job);
    int32_t finish(int32_t job);
    int32_t set_pending(int32_t job, uint64_t n);
    int32_t set_cost(int32_t job, uint64_t cost);
    int32_t query(int32_t job, salus_job_info *out) const;
    int32_t schedule(salus_slot *out, uint32_t cap, uint32_t *n);
    int32_t switch_out(int32_t job, void *pinned);
    int32_t switch_in(int32_t job);
    // Overlapped switching: begin_* decides and reserves, the caller moves the
    // bytes (host, offset, length are returned), end_* completes the bookkeeping.
    int32_t begin_out(int32_t job, void *pinned, void **host, uint64_t *off, uint64_t *len);
    int32_t end_out(int32_t job);
    int32_t begin_in(int32_t job, void **host, uint64_t *off, uint64_t *len);
    int32_t end_in(int32_t job);
    void drop_hold(int32_t job);     // a transfer failed: the job may now be freed (and only that)
    int32_t compact(std::vector<salus_move> *plan);

    const Job *job(int32_t id) const {
        return (id >= 0 && (size_t)id < jobs_.size()) ? &jobs_[id] : nullptr;
    }
    uint64_t lane_base(int32_t lane_id, uint64_t *size = nullptr) const;
    const std::vector<Lane> &lanes() const { return lanes_; }
    uint64_t capacity() const { return C_; }
    uint64_t floor() const { return C_ - sumL_; }
    uint64_t queued() const { return queue_.size(); }

    salus_stats stats{};
    std::vector<salus_event> events;
    std::string error;

private:
    enum Kind { NONE, NEW, USE, GROW };
    struct Choice { Kind kind = NONE; size_t index = 0; };

    // `gone`: per lane index, resident jobs to be counted as evicted (may be null)
    Choice find_lane(uint64_t P, uint64_t E, uint64_t residentP,
                     const std::vector<uint32_t> *gone = nullptr) const;
    bool can_restore(const Job &j) const;
    void left_device(Job &j);        // a resident job of a lane was evicted or finished
    size_t lane_index(int32_t lane_id) const;
    void process_requests();
    int admit(Job &j, Choice c);
    uint64_t entry_level(const Job &j) const;
    int place(Job &j, uint64_t fl);
    bool first_fit(uint64_t P, uint64_t fl, uint64_t *off) const;
    int evict(Job &j, bool automatic, void *pinned, bool copied = false);
    int host_buffer(Job &j, void *pinned);
    int32_t switch_in_impl(int32_t job, bool copy_now);
    int do_compact(std::vector<salus_move> *plan);
    void log(int32_t kind, uint64_t a, uint64_t b) { events.push_back({kind, 0, a, b}); }

    uint64_t C_, A_;
    uint32_t max_lanes_;
    int32_t policy_;
    bool shrink_lanes_;            // keep L_j == max E_i when a lane's largest job leaves
    DeviceOps *dev_;
    std::vector<Job> jobs_;
    std::vector<Lane> lanes_;             // creation order == address order from the top
    std::deque<int32_t> queue_;           // Q of Algorithm 1
    std::map<uint64_t, int32_t> blocks_;  // live persistent blocks: offset -> job
    uint64_t sumP_ = 0, sumL_ = 0;        // over resident jobs / over lanes that are not parked
    int32_t next_lane_ = 0;
    uint64_t round_ = 0;
};

}  // namespace salus
