// Depth-fused packed forward pass for gfx950 (MI355X): ONE launch runs every
// layer of every job scheduled in the round, instead of one launch per layer
// depth.  The Salus paper raises kernel batching and pipelining as the cost of
// scheduling below the iteration (Section 3.2.2); inside an iteration nothing
// forbids it, and it removes what the per-depth launches leave idle: the drain
// of one launch, the start of the next, and the uneven last wave of each depth.
//
// The grid holds the tiles of depth 0, then depth 1, ...  A tile of depth l > 0
// needs the whole activation H_l of its job, i.e. all tiles of (job, l - 1).
// Every (job, layer) pair of a launch has a completion counter in device memory:
// a workgroup adds one to its pair's counter after its stores are visible to the
// device, and a consumer waits until the producer pair's counter has reached
// that pair's tile count before it reads any activation.
//
// Why the wait ends: workgroups are handed to each XCD in ascending index order,
// and a depth's workgroups all have lower indices than the next depth's, so when
// a consumer is resident every producer on its XCD is resident or finished; the
// lowest unfinished depth anywhere never waits, hence always drains.  The wait is
// bounded all the same: after `spin_limit` polls the workgroup gives up, raises
// a host-visible flag and carries on (its output is then wrong, the flag says
// so), which means every wavefront of every launch exits.
//
// Descriptors do not fit the 4 KB of by-value kernel arguments (64 jobs x 3
// layers x 48 bytes), so they live in a device table that is rewritten only
// when a job's descriptor changes (a small kernel with by-value payload); what
// changes every round - which jobs run, their row counts, the tile ranges -
// travels by value.
#include <algorithm>
#include <cstring>
#include <vector>

#include "dense_tile.hpp"

namespace salus {

constexpr uint32_t kNone = 0xffffu;

struct ChainArgs {
    const Problem *table;      // device table, entry (job slot * kChainMaxLayers + layer)
    uint32_t *done;            // this launch's completion counters, all zero at its start
    uint32_t *clear;           // the other set: zeroed here for the launch that follows
    uint32_t *timed_out;       // host-visible word, set to 1 when a wait gives up
    uint32_t n_layers;
    uint32_t spin_limit;
    uint32_t layer_first[kChainMaxLayers + 1];   // first workgroup of each depth (multiples of 8)
    uint32_t pad;
    uint32_t first[kChainMaxProblems];   // first tile of pair i, ascending; unused entries ~0
    uint16_t slot[kChainMaxProblems];    // table entry of pair i; kNone: filler that ends a depth
    uint16_t M[kChainMaxProblems];       // rows of pair i's job in this round
    uint16_t dep[kChainMaxProblems];     // pair whose output pair i reads; kNone at depth 0
};
static_assert(sizeof(ChainArgs) <= 4096, "kernel arguments are limited to 4 KB");

struct ChainWork {
    Problem p;
    Tile tile;
    uint32_t pair, layer;
};

// Which pair and tile this workgroup owns.  Returns false for filler workgroups.
template <int TM, int TN>
__device__ inline bool chain_find(const ChainArgs &a, ChainWork &w)
{
    const int lane = threadIdx.x & 63;
    const uint32_t b = blockIdx.x;
    uint32_t l = 0;
    for (uint32_t i = 1; i < a.n_layers; ++i)
        if (b >= a.layer_first[i]) l = i;
    // XCD x (workgroups b with b % 8 == x) takes a contiguous eighth of the depth's tiles
    const uint32_t lo = a.layer_first[l], span = a.layer_first[l + 1] - lo, local = b - lo;
    const uint32_t id = lo + (local & 7u) * (span >> 3) + (local >> 3);

    // lane i looks at pairs 4i .. 4i+3; the last pair whose first tile is <= id owns it
    const uint32_t f0 = a.first[4 * lane], f1 = a.first[4 * lane + 1], f2 = a.first[4 * lane + 2],
                   f3 = a.first[4 * lane + 3];
    const uint32_t cnt = (f0 <= id) + (f1 <= id) + (f2 <= id) + (f3 <= id);
    const unsigned long long m = __ballot(f0 <= id);          // never empty: first[0] == 0
    const int owner = 63 - __clzll((long long)m);
    const uint32_t sel = cnt == 1 ? f0 : cnt == 2 ? f1 : cnt == 3 ? f2 : f3;
    const uint32_t start = __shfl(sel, owner, 64);
    const uint32_t pair = __builtin_amdgcn_readfirstlane(4 * owner + __shfl(cnt, owner, 64) - 1);
    const uint32_t slot = a.slot[pair];
    if (slot == kNone) return false;

    const uint32_t *e = (const uint32_t *)(a.table + slot);
    uint32_t d[12];
#pragma unroll
    for (int i = 0; i < 12; ++i) d[i] = __builtin_amdgcn_readfirstlane(e[i]);
    w.p.W = (const void *)(((uint64_t)d[1] << 32) | d[0]);
    w.p.X = (const void *)(((uint64_t)d[3] << 32) | d[2]);
    w.p.Y = (void *)(((uint64_t)d[5] << 32) | d[4]);
    w.p.aux = (const void *)(((uint64_t)d[7] << 32) | d[6]);
    w.p.M = a.M[pair];
    w.p.K = d[9];
    w.p.N = d[10];
    w.p.flags = d[11];
    const uint32_t t = id - start, rt = (w.p.M + TM - 1) / TM;
    w.tile.problem = (int)pair;
    w.tile.m0 = (t % rt) * TM;
    w.tile.n0 = (t / rt) * TN;
    w.pair = pair;
    w.layer = l;
    return true;
}
static_assert(sizeof(Problem) == 48, "the table is read as 12 dwords per entry");

// Block until every tile of the producer pair has been stored (or give up after
// spin_limit polls).  One wavefront polls and then acquires at device scope, which
// drops what this CU and this XCD's L2 cached of other XCDs' memory; the barrier
// hands that on to the other three (they share the CU's cache).
__device__ inline void chain_wait(const ChainArgs &a, uint32_t pair)
{
    const uint32_t dep = a.dep[pair];
    if (dep == kNone) return;
    if (threadIdx.x < 64) {
        const uint32_t target = a.first[dep + 1] - a.first[dep];
        uint32_t polls = 0;
        while (__hip_atomic_load(a.done + dep, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            if (polls++ >= a.spin_limit) {
                if (threadIdx.x == 0)
                    __hip_atomic_store(a.timed_out, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                break;
            }
            __builtin_amdgcn_s_sleep(32);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    __syncthreads();
}

// Count the tile once its stores are visible to the device.  Every wavefront
// waits for its own stores to reach the L2 (release at workgroup scope), the
// barrier orders them before the first wavefront's release at device scope, whose
// L2 write-back then covers all four: a quarter of the cache operations that a
// device-scope release in every wavefront costs (the write-back is what makes
// this launch slow).
__device__ inline void chain_signal(const ChainArgs &a, uint32_t pair)
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0x0f70);       // vmcnt(0): this wavefront's stores are in the L2
    __syncthreads();
    if (threadIdx.x == 0)
        __hip_atomic_fetch_add(a.done + pair, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

template <bool BF16, int MT>
__global__ __launch_bounds__(kGemmThreads) void chained_dense(ChainArgs a)
{
    constexpr int NACC = MT * (BF16 ? 8 : 4);
    __shared__ float lds[reduce_lds_floats<NACC>()];
    if (blockIdx.x == 0) a.clear[threadIdx.x] = 0u;       // kChainMaxProblems == workgroup size
    ChainWork w;
    if (!chain_find<16 * MT, BF16 ? 128 : 64>(a, w)) return;
    chain_wait(a, w.pair);
    if (BF16) dense_bf16_tile<MT, false, true>(w.p, w.tile, lds);   // at most 32 rows: one row tile
    else dense_f32_tile<MT>(w.p, w.tile, lds);
    if (w.layer + 1 < a.n_layers) chain_signal(a, w.pair);
}
static_assert(kChainMaxProblems == (uint32_t)kGemmThreads, "one thread clears one counter");

constexpr uint32_t kWriteMax = 48;
struct TableWrite {
    Problem *table;
    uint32_t n;
    uint32_t slot[kWriteMax];
    Problem p[kWriteMax];
};
static_assert(sizeof(TableWrite) <= 4096, "kernel arguments are limited to 4 KB");

__global__ __launch_bounds__(64) void chain_table_write(TableWrite a)
{
    const uint32_t i = threadIdx.x;
    if (i < a.n) a.table[a.slot[i]] = a.p[i];
}

// ---------------------------------------------------------------------------
struct Chain {
    Problem *table = nullptr;          // device, kChainJobSlots * kChainMaxLayers entries
    uint32_t *banks = nullptr;         // device, two sets of kChainMaxProblems counters
    uint32_t *flag = nullptr;          // pinned host word the kernels raise
    uint32_t *flag_dev = nullptr;      // its device address
    int bank = 0;
    uint64_t stamp = 0;                // launches so far
    std::vector<Problem> mirror;       // what the device table holds
    std::vector<int64_t> slot_key;     // job cached in each slot (-1: none)
    std::vector<uint64_t> slot_stamp;  // launch that used the slot last
};

hipError_t chain_create(Chain **out)
{
    Chain *c = new Chain;
    const size_t entries = (size_t)kChainJobSlots * kChainMaxLayers;
    hipError_t e = hipMalloc((void **)&c->table, entries * sizeof(Problem));
    if (e == hipSuccess) e = hipMalloc((void **)&c->banks, 2 * kChainMaxProblems * sizeof(uint32_t));
    if (e == hipSuccess) e = hipMemset(c->banks, 0, 2 * kChainMaxProblems * sizeof(uint32_t));
    if (e == hipSuccess) e = hipMemset(c->table, 0, entries * sizeof(Problem));
    if (e == hipSuccess) e = hipHostMalloc((void **)&c->flag, sizeof(uint32_t), hipHostMallocMapped);
    if (e == hipSuccess) e = hipHostGetDevicePointer((void **)&c->flag_dev, c->flag, 0);
    if (e != hipSuccess) {
        chain_destroy(c);
        return e;
    }
    *c->flag = 0;
    c->mirror.assign(entries, Problem{});
    c->slot_key.assign(kChainJobSlots, -1);
    c->slot_stamp.assign(kChainJobSlots, 0);
    *out = c;
    return hipSuccess;
}

void chain_destroy(Chain *c)
{
    if (!c) return;
    if (c->table) (void)hipFree(c->table);
    if (c->banks) (void)hipFree(c->banks);
    if (c->flag) (void)hipHostFree(c->flag);
    delete c;
}

uint32_t chain_take_timeouts(Chain *c)
{
    const uint32_t v = *(volatile uint32_t *)c->flag;
    *(volatile uint32_t *)c->flag = 0;
    return v;
}

static uint32_t job_slot(Chain *c, int64_t key)
{
    uint32_t lru = 0;
    for (uint32_t s = 0; s < kChainJobSlots; ++s) {
        if (c->slot_key[s] == key) {
            c->slot_stamp[s] = c->stamp;
            return s;
        }
        if (c->slot_stamp[s] < c->slot_stamp[lru]) lru = s;
    }
    // a launch names at most kChainJobSlots jobs, so the least recently used slot
    // belongs to none of this launch's jobs
    c->slot_key[lru] = key;
    c->slot_stamp[lru] = c->stamp;
    return lru;
}

static hipError_t launch_one(Chain *c, const ChainJob *jobs, uint32_t n, bool bf16, uint32_t spin_limit,
                             hipStream_t stream)
{
    c->stamp += 1;
    ChainArgs a{};
    uint32_t depth = 0, max_m = 0;
    for (uint32_t i = 0; i < n; ++i) {
        depth = std::max(depth, jobs[i].n_layers);
        max_m = std::max(max_m, jobs[i].M);
    }
    const int mt = max_m <= 16 ? 1 : (bf16 || max_m <= 32) ? 2 : 4;
    const uint32_t tm = 16u * mt, tn = bf16 ? 128u : 64u;
    std::fill(a.first, a.first + kChainMaxProblems, ~0u);
    std::vector<uint32_t> slot_of(n), prev(n, kNone);
    for (uint32_t i = 0; i < n; ++i) slot_of[i] = job_slot(c, jobs[i].key);

    TableWrite tw{};
    tw.table = c->table;
    auto flush = [&]() {
        if (tw.n) hipLaunchKernelGGL(chain_table_write, dim3(1), dim3(64), 0, stream, tw);
        tw.n = 0;
    };
    uint32_t pairs = 0;
    uint64_t running = 0;
    for (uint32_t l = 0; l < depth; ++l) {
        a.layer_first[l] = (uint32_t)running;
        for (uint32_t i = 0; i < n; ++i) {
            if (l >= jobs[i].n_layers) continue;
            Problem p = jobs[i].layer[l];
            p.M = 0;                                   // rows travel by value
            const uint32_t entry = slot_of[i] * kChainMaxLayers + l;
            if (std::memcmp(&c->mirror[entry], &p, sizeof(Problem)) != 0) {
                c->mirror[entry] = p;
                tw.slot[tw.n] = entry;
                tw.p[tw.n] = p;
                if (++tw.n == kWriteMax) flush();
            }
            a.first[pairs] = (uint32_t)running;
            a.slot[pairs] = (uint16_t)entry;
            a.M[pairs] = (uint16_t)jobs[i].M;
            a.dep[pairs] = (uint16_t)prev[i];
            prev[i] = pairs++;
            running += (uint64_t)((jobs[i].M + tm - 1) / tm) * ((p.N + tn - 1) / tn);
        }
        // the filler rounds the depth up to a multiple of 8 workgroups, so that a
        // workgroup's XCD is its index within the depth modulo 8
        a.first[pairs] = (uint32_t)running;
        a.slot[pairs] = (uint16_t)kNone;
        a.dep[pairs] = (uint16_t)kNone;
        ++pairs;
        running = (running + 7) & ~(uint64_t)7;
        if (running > 0x7fffffffull) return hipErrorInvalidValue;
    }
    a.layer_first[depth] = (uint32_t)running;
    flush();
    a.table = c->table;
    a.done = c->banks + (size_t)c->bank * kChainMaxProblems;
    a.clear = c->banks + (size_t)(c->bank ^ 1) * kChainMaxProblems;
    c->bank ^= 1;
    a.timed_out = c->flag_dev;
    a.n_layers = depth;
    a.spin_limit = spin_limit;
    const dim3 grid((uint32_t)running), block(kGemmThreads);
    if (bf16) {
        if (mt == 1) hipLaunchKernelGGL((chained_dense<true, 1>), grid, block, 0, stream, a);
        else hipLaunchKernelGGL((chained_dense<true, 2>), grid, block, 0, stream, a);
    } else {
        if (mt == 1) hipLaunchKernelGGL((chained_dense<false, 1>), grid, block, 0, stream, a);
        else if (mt == 2) hipLaunchKernelGGL((chained_dense<false, 2>), grid, block, 0, stream, a);
        else hipLaunchKernelGGL((chained_dense<false, 4>), grid, block, 0, stream, a);
    }
    return hipGetLastError();
}

hipError_t launch_chain(Chain *c, const ChainJob *jobs, uint32_t n, bool bf16, uint32_t spin_limit,
                        hipStream_t stream, uint64_t *launches)
{
    uint32_t at = 0;
    while (at < n) {
        // as many jobs as the job slots and the pair table hold (one filler per depth)
        uint32_t count = 0, pairs = 0, depth = 0;
        while (at + count < n && count < kChainJobSlots) {
            const ChainJob &j = jobs[at + count];
            if (j.n_layers == 0 || j.n_layers > kChainMaxLayers || j.M == 0 || j.M > 0xffffu)
                return hipErrorInvalidValue;
            const uint32_t d = std::max(depth, j.n_layers);
            if (pairs + j.n_layers + d > kChainMaxProblems) break;
            pairs += j.n_layers;
            depth = d;
            ++count;
        }
        hipError_t e = launch_one(c, jobs + at, count, bf16, spin_limit, stream);
        if (e != hipSuccess) return e;
        if (launches) *launches += 1;
        at += count;
    }
    return hipSuccess;
}

}  // namespace salus
