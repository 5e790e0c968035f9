// C ABI of the library (declared in include/salus.h): argument checking, the
// HIP implementation of the data-movement interface the host logic uses, and
// the translation of job descriptors into grouped-GEMM problem lists.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <map>
#include <memory>
#include <new>
#include <string>
#include <vector>

#include "device.hpp"
#include "pool_core.hpp"
#include "salus.h"

using namespace salus;

namespace {

struct HipOps : DeviceOps {
    char *base = nullptr;
    uint64_t capacity = 0;
    hipStream_t stream = nullptr;
    int engine = SALUS_COPY_KERNEL;
    std::string *error = nullptr;
    uint64_t copy_launches = 0;
    SlideState slide_state;                 // counters of the in-place compaction kernel (16 KB on the device)
    // transfers begun and not yet ended (job id -> fence on the pool's stream, completion event)
    struct Transfer { hipEvent_t fence, done; bool failed; };
    std::map<int32_t, Transfer> inflight;

    bool present() const override { return base != nullptr; }

    int fail(hipError_t e, const char *what)
    {
        if (error) *error = std::string(what) + ": " + hipGetErrorString(e);
        return -1;
    }

    int host_copy(void *dst, const void *src, uint64_t n, hipMemcpyKind kind)
    {
        if (n == 0) return 0;
        hipError_t e;
        if (engine == SALUS_COPY_KERNEL) {
            // the kernel reads / writes the pinned buffer through its device mapping
            void *mapped = nullptr;
            void *host = kind == hipMemcpyDeviceToHost ? dst : const_cast<void *>(src);
            e = hipHostGetDevicePointer(&mapped, host, 0);
            if (e != hipSuccess) return fail(e, "hipHostGetDevicePointer");
            CopySeg seg = kind == hipMemcpyDeviceToHost ? CopySeg{src, mapped, n}
                                                        : CopySeg{mapped, dst, n};
            e = launch_copy(&seg, 1, stream);
            copy_launches += 1;
        } else {
            e = hipMemcpyAsync(dst, src, n, kind, stream);
        }
        if (e != hipSuccess) return fail(e, "host link copy");
        e = hipStreamSynchronize(stream);
        if (e != hipSuccess) return fail(e, "hipStreamSynchronize");
        return 0;
    }

    int evict(void *host, uint64_t off, uint64_t n) override
    {
        return host_copy(host, base + off, n, hipMemcpyDeviceToHost);
    }
    int restore(uint64_t off, const void *host, uint64_t n) override
    {
        return host_copy(base + off, host, n, hipMemcpyHostToDevice);
    }
    int slide(const salus_move *m, uint32_t n) override
    {
        std::vector<uint64_t> s(n), d(n), l(n);
        for (uint32_t i = 0; i < n; ++i) { s[i] = m[i].src; d[i] = m[i].dst; l[i] = m[i].len; }
        // blocks with a transfer in flight may be among those that move: the moves
        // are ordered after every such transfer
        for (const auto &kv : inflight) {
            hipError_t w = hipStreamWaitEvent(stream, kv.second.done, 0);
            if (w != hipSuccess) return fail(w, "hipStreamWaitEvent");
        }
        hipError_t e = launch_slide(base, s.data(), d.data(), l.data(), n, &slide_state, stream, &copy_launches);
        if (e != hipSuccess) return fail(e, "compaction launch");
        uint32_t gave_up = 0;
        e = slide_state_failed(&slide_state, stream, &gave_up);       // synchronizes the stream
        if (e != hipSuccess) return fail(e, "hipStreamSynchronize");
        if (gave_up) {
            if (error) *error = "an in-place move gave up waiting for a neighbouring chunk: the persistent region is damaged";
            return -1;
        }
        return 0;
    }
    void *pinned_alloc(uint64_t n) override
    {
        void *p = nullptr;
        if (hipHostMalloc(&p, n, hipHostMallocMapped | hipHostMallocPortable) != hipSuccess) return nullptr;
        return p;
    }
    void pinned_free(void *p) override { (void)hipHostFree(p); }
};

}  // namespace

struct salus_pool {
    HipOps ops;
    std::unique_ptr<PoolCore> core;
    std::string error;
    std::string device_error;               // written by the device layer underneath a pool operation
    uint64_t granule = 256;
    uint64_t gemm_launches = 0;
    Chain *chain = nullptr;                 // SALUS_FLAG_FUSE_DEPTHS: the depth-fused forward's device state
    uint32_t spin_limit = kChainSpinLimit;
    uint64_t fused_timeouts = 0;
};

#define CHECK_POOL(p) \
    if (!(p)) return SALUS_EINVAL

// Hidden activations of salus_grouped_forward_static.  Every GPU the library runs
// on holds its own copy of this array until the process ends.  In host code the
// name below is only a handle for hipGetSymbolAddress, never a device address:
// host code uses the per-device pointer obtained in static_scratch().
constexpr uint64_t kStaticScratchBytes = SALUS_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static char *g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device (looked up once per device).
static hipError_t static_scratch(char **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = (char *)ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

static int32_t set_error(salus_pool *p, int32_t code, const std::string &msg)
{
    p->error = msg;
    return code;
}

static int32_t done(salus_pool *p, int32_t rc)
{
    if (rc < 0 && !p->core->error.empty()) {
        p->error = p->core->error;
        // what the device layer said about the same failure is the more specific half
        if (!p->device_error.empty()) p->error += " (" + p->device_error + ")";
    }
    p->device_error.clear();
    return rc;
}

extern "C" {

int32_t salus_pool_create(void *base, uint64_t capacity, const salus_config *cfg, salus_pool_t **out)
{
    if (!out) return SALUS_EINVAL;
    *out = nullptr;
    salus_config c{};
    if (cfg) c = *cfg;
    if (c.granule == 0) c.granule = 256;
    if (c.granule < 16 || (c.granule & (c.granule - 1))) return SALUS_EINVAL;
    if (capacity == 0 || capacity % c.granule) return SALUS_EINVAL;
    if ((uintptr_t)base % 256) return SALUS_EINVAL;
    if (c.policy < SALUS_POLICY_FIFO || c.policy > SALUS_POLICY_PACK) return SALUS_EINVAL;
    if (c.copy_engine != SALUS_COPY_KERNEL && c.copy_engine != SALUS_COPY_DMA) return SALUS_EINVAL;
    salus_pool *p = new (std::nothrow) salus_pool;
    if (!p) return SALUS_ENOMEM;
    p->ops.base = (char *)base;
    p->ops.capacity = capacity;
    p->ops.stream = (hipStream_t)c.stream;
    p->ops.engine = c.copy_engine;
    p->ops.error = &p->device_error;
    p->granule = c.granule;
    p->core.reset(new PoolCore(capacity, c.granule, c.max_lanes, c.policy,
                               (c.flags & SALUS_FLAG_SHRINK_LANES) != 0, &p->ops));
    if (base && slide_state_create(&p->ops.slide_state) != hipSuccess) {
        delete p;
        return SALUS_EHIP;
    }
    if ((c.flags & SALUS_FLAG_FUSE_DEPTHS) && base) {
        if (chain_create(&p->chain) != hipSuccess) {
            slide_state_destroy(&p->ops.slide_state);
            delete p;
            return SALUS_EHIP;
        }
    }
    *out = p;
    return SALUS_OK;
}

int32_t salus_pool_destroy(salus_pool_t *pool)
{
    CHECK_POOL(pool);
    for (auto &kv : pool->ops.inflight) {     // let unfinished transfers land before their buffers go
        (void)hipEventSynchronize(kv.second.done);
        (void)hipEventDestroy(kv.second.fence);
        (void)hipEventDestroy(kv.second.done);
    }
    pool->ops.inflight.clear();
    if (pool->chain) {
        (void)hipDeviceSynchronize();         // no launch may still read the table
        chain_destroy(pool->chain);
    }
    slide_state_destroy(&pool->ops.slide_state);
    delete pool;
    return SALUS_OK;
}

int32_t salus_lane_alloc(salus_pool_t *pool, uint64_t P, uint64_t E, int32_t priority,
                         uint64_t pending, int32_t *job)
{
    CHECK_POOL(pool);
    return done(pool, pool->core->arrive(P, E, priority, pending, job));
}

int32_t salus_lane_free(salus_pool_t *pool, int32_t job)
{
    CHECK_POOL(pool);
    // a job whose transfer failed can only be given up: its hold is dropped here
    auto it = pool->ops.inflight.find(job);
    if (it != pool->ops.inflight.end() && it->second.failed) {
        (void)hipEventDestroy(it->second.fence);
        (void)hipEventDestroy(it->second.done);
        pool->ops.inflight.erase(it);
        pool->core->drop_hold(job);
    }
    return done(pool, pool->core->finish(job));
}

int32_t salus_job_query(salus_pool_t *pool, int32_t job, salus_job_info *out)
{
    CHECK_POOL(pool);
    int32_t rc = pool->core->query(job, out);
    if (rc) return set_error(pool, rc, "no such job");
    return rc;
}

int32_t salus_job_set_pending(salus_pool_t *pool, int32_t job, uint64_t n)
{
    CHECK_POOL(pool);
    return done(pool, pool->core->set_pending(job, n));
}

int32_t salus_job_set_cost(salus_pool_t *pool, int32_t job, uint64_t cost)
{
    CHECK_POOL(pool);
    return done(pool, pool->core->set_cost(job, cost));
}

int32_t salus_set_pending_many(salus_pool_t *pool, const int32_t *jobs, const uint64_t *n,
                               uint32_t count)
{
    CHECK_POOL(pool);
    if (count && (!jobs || !n)) return set_error(pool, SALUS_EINVAL, "null array");
    for (uint32_t i = 0; i < count; ++i)
        if (int32_t rc = pool->core->set_pending(jobs[i], n[i])) return done(pool, rc);
    return SALUS_OK;
}

static int32_t job_io(salus_pool *pool, int32_t job, uint64_t off, void *host, uint64_t n, bool write)
{
    const Job *j = pool->core->job(job);
    if (!j || !host) return set_error(pool, SALUS_EINVAL, "bad job or buffer");
    if (j->state != SALUS_JOB_RESIDENT) return set_error(pool, SALUS_ENOTRESIDENT, "job is not resident");
    if (j->held) return set_error(pool, SALUS_EBUSY, "job is in transit");
    if (off > j->P || n > j->P - off) return set_error(pool, SALUS_EINVAL, "range outside the persistent block");
    if (!pool->ops.present()) return set_error(pool, SALUS_EINVAL, "pool has no device memory");
    char *dev = pool->ops.base + j->off + off;
    hipError_t e = write ? hipMemcpyAsync(dev, host, n, hipMemcpyHostToDevice, pool->ops.stream)
                         : hipMemcpyAsync(host, dev, n, hipMemcpyDeviceToHost, pool->ops.stream);
    if (e == hipSuccess) e = hipStreamSynchronize(pool->ops.stream);
    if (e != hipSuccess) return set_error(pool, SALUS_EHIP, hipGetErrorString(e));
    return SALUS_OK;
}

int32_t salus_job_write(salus_pool_t *pool, int32_t job, uint64_t off, const void *host_src,
                        uint64_t nbytes)
{
    CHECK_POOL(pool);
    return job_io(pool, job, off, const_cast<void *>(host_src), nbytes, true);
}

int32_t salus_job_read(salus_pool_t *pool, int32_t job, uint64_t off, void *host_dst, uint64_t nbytes)
{
    CHECK_POOL(pool);
    return job_io(pool, job, off, host_dst, nbytes, false);
}

int32_t salus_schedule_iteration(salus_pool_t *pool, salus_slot *out, uint32_t cap, uint32_t *n)
{
    CHECK_POOL(pool);
    return done(pool, pool->core->schedule(out, cap, n));
}

static bool overlap(uint64_t a, uint64_t an, uint64_t b, uint64_t bn)
{
    return an && bn && a < b + bn && b < a + an;
}

static uint64_t up256(uint64_t v) { return (v + 255) & ~(uint64_t)255; }

// Scratch of a forward pass inside the lane: two row-major buffers of M x (widest
// hidden layer) that the layers write and read alternately.
static void forward_scratch(uint32_t M, const salus_layer *layers, uint32_t n_layers, int32_t dtype,
                            uint64_t *xp_bytes, uint64_t *h_stride)
{
    uint32_t max_n = 0;
    for (uint32_t l = 0; l + 1 < n_layers; ++l) max_n = std::max(max_n, layers[l].N);
    *xp_bytes = 0;
    if (dtype == SALUS_BF16 && M <= kBlockedMaxM) {
        // blocked order: whole 16-row tiles and whole 32-column k-steps
        *h_stride = up256((uint64_t)((M + 15) / 16 * 16) * ((max_n + 31) / 32 * 32) * 2);
        return;
    }
    *h_stride = up256((uint64_t)M * max_n * (dtype == SALUS_BF16 ? 2 : 4));
}

uint64_t salus_forward_work_bytes(uint32_t M, const salus_layer *layers, uint32_t n_layers, int32_t dtype)
{
    if (!layers || n_layers == 0 || M == 0) return 0;
    uint64_t xp, hs;
    forward_scratch(M, layers, n_layers, dtype, &xp, &hs);
    return xp + (n_layers > 1 ? 2 * hs : 0);
}

// hidden == nullptr: the hidden activations live at h_off inside each job's lane.
// Otherwise they are carved out of [hidden, hidden + hidden_bytes), h_off is
// ignored and the depth-fused path is not taken.
static int32_t forward_impl(salus_pool_t *pool, const salus_gemm_desc *descs, uint32_t n,
                            void *stream, char *hidden, uint64_t hidden_bytes)
{
    if (n == 0) return SALUS_OK;
    if (!descs) return set_error(pool, SALUS_EINVAL, "null descriptor array");
    if (!pool->ops.present()) return set_error(pool, SALUS_EINVAL, "pool has no device memory");
    char *base = pool->ops.base;
    uint32_t depth = 0;
    uint64_t hidden_used = 0;
    std::vector<int32_t> lanes_used;
    struct Resolved { char *w, *x, *y, *xp, *h; uint64_t hstride; };
    std::vector<Resolved> res(n);
    for (uint32_t i = 0; i < n; ++i) {
        const salus_gemm_desc &d = descs[i];
        const Job *j = pool->core->job(d.job);
        if (!j) return set_error(pool, SALUS_EINVAL, "descriptor names an unknown job");
        if (j->state != SALUS_JOB_RESIDENT)
            return set_error(pool, SALUS_ENOTRESIDENT, "job " + std::to_string(d.job) + " is not resident");
        if (j->held)
            return set_error(pool, SALUS_EBUSY, "job " + std::to_string(d.job) + " is in transit");
        if (std::find(lanes_used.begin(), lanes_used.end(), j->lane) != lanes_used.end())
            return set_error(pool, SALUS_EBUSY, "two jobs of lane " + std::to_string(j->lane) +
                                                    " in one packed iteration");
        lanes_used.push_back(j->lane);
        if (d.dtype != SALUS_F32 && d.dtype != SALUS_BF16) return set_error(pool, SALUS_EINVAL, "bad dtype");
        if (d.n_layers == 0 || !d.layers || d.M == 0) return set_error(pool, SALUS_EINVAL, "empty job descriptor");
        const uint32_t esz = d.dtype == SALUS_BF16 ? 2 : 4;
        const uint32_t mult = 16 / esz;
        uint64_t lane_size = 0;
        const uint64_t lane_off = pool->core->lane_base(j->lane, &lane_size);
        for (uint32_t l = 0; l < d.n_layers; ++l) {
            const salus_layer &L = d.layers[l];
            if (L.K == 0 || L.N == 0 || L.K % mult || L.N % mult)
                return set_error(pool, SALUS_EINVAL, "K and N must be positive multiples of 16 bytes");
            if (l && L.K != d.layers[l - 1].N) return set_error(pool, SALUS_EINVAL, "layer widths do not chain");
            if (L.act < SALUS_ACT_NONE || L.act > SALUS_ACT_GELU) return set_error(pool, SALUS_EINVAL, "bad activation");
            if (L.layout != SALUS_LAYOUT_ROWMAJOR &&
                (L.layout != SALUS_LAYOUT_STRIP128 || d.dtype != SALUS_BF16 || L.N % 128))
                return set_error(pool, SALUS_EINVAL, "strip layout needs bf16 weights and N a multiple of 128");
            const uint64_t wbytes = (uint64_t)L.K * L.N * esz;
            if (L.w_off % 16 || L.w_off > j->P || wbytes > j->P - L.w_off)
                return set_error(pool, SALUS_EINVAL, "weights outside the persistent block");
        }
        const uint64_t xbytes = (uint64_t)d.M * d.layers[0].K * esz;
        const uint64_t ybytes = (uint64_t)d.M * d.layers[d.n_layers - 1].N * 4;
        uint64_t xp_bytes, hstride;
        forward_scratch(d.M, d.layers, d.n_layers, d.dtype, &xp_bytes, &hstride);
        const uint64_t hbytes = xp_bytes + (d.n_layers > 1 ? 2 * hstride : 0);
        auto inside = [&](uint64_t off, uint64_t nb) { return off % 16 == 0 && off <= lane_size && nb <= lane_size - off; };
        if (!inside(d.x_off, xbytes) || !inside(d.y_off, ybytes) || (!hidden && !inside(d.h_off, hbytes)))
            return set_error(pool, SALUS_EINVAL, "buffer outside the job's lane");
        if (overlap(d.x_off, xbytes, d.y_off, ybytes) ||
            (!hidden && (overlap(d.x_off, xbytes, d.h_off, hbytes) || overlap(d.y_off, ybytes, d.h_off, hbytes))))
            return set_error(pool, SALUS_EINVAL, "x, y and h ranges overlap");
        char *lane = base + lane_off;
        char *h = lane + d.h_off;
        if (hidden) {
            if (hbytes > hidden_bytes - hidden_used)
                return set_error(pool, SALUS_ENOMEM,
                                 "the hidden activations of this round exceed the static scratch of " +
                                     std::to_string(hidden_bytes) + " bytes");
            h = hidden + hidden_used;
            hidden_used += up256(hbytes);
            if (hidden_used > hidden_bytes) hidden_used = hidden_bytes;
        }
        res[i] = {base + j->off, lane + d.x_off, lane + d.y_off, h, h + xp_bytes, hstride};
        depth = std::max(depth, d.n_layers);
    }
    hipStream_t s = (hipStream_t)stream;
    auto problem = [&](uint32_t i, uint32_t l) {
        const salus_gemm_desc &d = descs[i];
        const salus_layer &L = d.layers[l];
        const bool last = l + 1 == d.n_layers;
        const bool bf = d.dtype == SALUS_BF16;
        Problem pr{};
        pr.W = res[i].w + L.w_off;
        pr.X = l == 0 ? res[i].x : res[i].h + ((l - 1) & 1) * res[i].hstride;
        pr.Y = last ? res[i].y : res[i].h + (l & 1) * res[i].hstride;
        pr.M = d.M;
        pr.K = L.K;
        pr.N = L.N;
        pr.flags = (uint32_t)L.act;
        if (bf && !last) pr.flags |= kOutBf16;
        if (L.layout == SALUS_LAYOUT_STRIP128) pr.flags |= kStripW;
        if (bf && d.M <= kBlockedMaxM) {      // hidden activations in MFMA operand order
            if (l > 0) pr.flags |= kInBlocked;
            if (!last) pr.flags |= kOutBlocked;
        }
        return pr;
    };
    std::vector<Problem> probs;
    for (int dt = SALUS_F32; dt <= SALUS_BF16; ++dt) {
        // Depth-fused: all layers of all jobs of this type in one launch, if every
        // job is one the weight-streaming kernels take (bf16: at most 32 rows).
        if (pool->chain && !hidden) {
            bool fits = true, any = false;
            for (uint32_t i = 0; i < n && fits; ++i) {
                const salus_gemm_desc &d = descs[i];
                if (d.dtype != dt) continue;
                any = true;
                fits = d.n_layers <= kChainMaxLayers && d.M <= (dt == SALUS_BF16 ? kBlockedMaxM : 0xffffu);
            }
            if (any && fits) {
                // its two sets of counters alternate from launch to launch, which a
                // replayed recording would not do
                hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
                if (hipStreamIsCapturing(s, &capturing) != hipSuccess || capturing != hipStreamCaptureStatusNone)
                    return set_error(pool, SALUS_EINVAL, "the depth-fused forward cannot be recorded in a graph");
                std::vector<ChainJob> jobs;
                for (uint32_t i = 0; i < n; ++i) {
                    const salus_gemm_desc &d = descs[i];
                    if (d.dtype != dt) continue;
                    ChainJob cj{};
                    cj.key = d.job;
                    cj.M = d.M;
                    cj.n_layers = d.n_layers;
                    for (uint32_t l = 0; l < d.n_layers; ++l) cj.layer[l] = problem(i, l);
                    jobs.push_back(cj);
                }
                hipError_t e = launch_chain(pool->chain, jobs.data(), (uint32_t)jobs.size(), dt == SALUS_BF16,
                                            pool->spin_limit, s, &pool->gemm_launches);
                if (e != hipSuccess) return set_error(pool, SALUS_EHIP, hipGetErrorString(e));
                continue;
            }
        }
        // one grouped launch per layer depth over all jobs that have that layer
        for (uint32_t l = 0; l < depth; ++l) {
            probs.clear();
            for (uint32_t i = 0; i < n; ++i)
                if (descs[i].dtype == dt && l < descs[i].n_layers) probs.push_back(problem(i, l));
            if (probs.empty()) continue;
            hipError_t e = dt == SALUS_BF16
                               ? launch_grouped_bf16(probs.data(), (uint32_t)probs.size(), false, s, &pool->gemm_launches)
                               : launch_grouped_f32(probs.data(), (uint32_t)probs.size(), s, &pool->gemm_launches);
            if (e != hipSuccess) return set_error(pool, SALUS_EHIP, hipGetErrorString(e));
        }
    }
    return SALUS_OK;
}

int32_t salus_grouped_forward(salus_pool_t *pool, const salus_gemm_desc *descs, uint32_t n,
                              void *stream)
{
    CHECK_POOL(pool);
    return forward_impl(pool, descs, n, stream, nullptr, 0);
}

int32_t salus_grouped_forward_static(salus_pool_t *pool, const salus_gemm_desc *descs, uint32_t n,
                                     void *stream)
{
    CHECK_POOL(pool);
    char *ptr = nullptr;
    hipError_t e = static_scratch(&ptr);
    if (e != hipSuccess)
        return set_error(pool, SALUS_EHIP, std::string("static scratch: ") + hipGetErrorString(e));
    return forward_impl(pool, descs, n, stream, ptr, kStaticScratchBytes);
}

int32_t salus_fused_check(salus_pool_t *pool)
{
    CHECK_POOL(pool);
    if (!pool->chain) return SALUS_OK;
    if (chain_take_timeouts(pool->chain) == 0) return SALUS_OK;
    pool->fused_timeouts += 1;
    return set_error(pool, SALUS_ETIMEOUT, "a depth-fused forward gave up waiting for a layer's input; "
                                            "the outputs of the launches since the last check are invalid");
}

int32_t salus_fused_spin_limit(salus_pool_t *pool, uint32_t polls)
{
    CHECK_POOL(pool);
    pool->spin_limit = polls;
    return SALUS_OK;
}

int32_t salus_compact_spin_limit(salus_pool_t *pool, uint32_t polls)
{
    CHECK_POOL(pool);
    pool->ops.slide_state.spin_limit = polls;
    return SALUS_OK;
}

// Scratch layout of a training step inside the lane: H_1 .. H_{L-1} (bf16, kept
// for the backward pass), then one gradient buffer of M x max_l(N_l) bf16 per layer
// (at least two): every layer's incoming gradient stays until the single launch
// at the end of the step that updates all layers.
uint64_t salus_train_work_bytes(uint32_t M, const salus_train_layer *layers, uint32_t n_layers)
{
    if (!layers || n_layers == 0) return 0;
    uint64_t total = 0, max_n = 0;
    for (uint32_t l = 0; l < n_layers; ++l) {
        if (l + 1 < n_layers) total += up256((uint64_t)M * layers[l].N * 2);
        max_n = std::max<uint64_t>(max_n, layers[l].N);
    }
    return total + std::max<uint64_t>(n_layers, 2) * up256((uint64_t)M * max_n * 2);
}

int32_t salus_grouped_train_step(salus_pool_t *pool, const salus_train_desc *descs, uint32_t n,
                                 void *stream_)
{
    CHECK_POOL(pool);
    if (n == 0) return SALUS_OK;
    if (!descs) return set_error(pool, SALUS_EINVAL, "null descriptor array");
    if (!pool->ops.present()) return set_error(pool, SALUS_EINVAL, "pool has no device memory");
    hipStream_t stream = (hipStream_t)stream_;
    char *base = pool->ops.base;
    struct Resolved {
        char *persist, *lane;
        std::vector<uint64_t> h_off;   // lane offset of H_l, l = 0 (= x) .. L-1
        std::vector<uint64_t> g_off;   // gradient buffer of backward step 0 .. L-1 (at least two)
    };
    std::vector<Resolved> res(n);
    std::vector<int32_t> lanes_used;
    uint32_t depth = 0;
    for (uint32_t i = 0; i < n; ++i) {
        const salus_train_desc &d = descs[i];
        const Job *j = pool->core->job(d.job);
        if (!j) return set_error(pool, SALUS_EINVAL, "descriptor names an unknown job");
        if (j->state != SALUS_JOB_RESIDENT)
            return set_error(pool, SALUS_ENOTRESIDENT, "job " + std::to_string(d.job) + " is not resident");
        if (j->held)
            return set_error(pool, SALUS_EBUSY, "job " + std::to_string(d.job) + " is in transit");
        if (std::find(lanes_used.begin(), lanes_used.end(), j->lane) != lanes_used.end())
            return set_error(pool, SALUS_EBUSY, "two jobs of lane " + std::to_string(j->lane) +
                                                    " in one packed iteration");
        lanes_used.push_back(j->lane);
        if (d.n_layers == 0 || !d.layers || d.M == 0) return set_error(pool, SALUS_EINVAL, "empty job descriptor");
        uint64_t lane_size = 0;
        const uint64_t lane_off = pool->core->lane_base(j->lane, &lane_size);
        for (uint32_t l = 0; l < d.n_layers; ++l) {
            const salus_train_layer &L = d.layers[l];
            if (L.K == 0 || L.N == 0 || L.K % 8 || L.N % 8)
                return set_error(pool, SALUS_EINVAL, "K and N must be positive multiples of 8");
            if (l && L.K != d.layers[l - 1].N) return set_error(pool, SALUS_EINVAL, "layer widths do not chain");
            const uint64_t elems = (uint64_t)L.K * L.N;
            if (L.wb_off % 16 || L.wb_off > j->P || elems * 2 > j->P - L.wb_off || L.wm_off % 16 ||
                L.wm_off > j->P || elems * 4 > j->P - L.wm_off)
                return set_error(pool, SALUS_EINVAL, "weights outside the persistent block");
            if (overlap(L.wb_off, elems * 2, L.wm_off, elems * 4))
                return set_error(pool, SALUS_EINVAL, "working and master weights overlap");
        }
        const uint32_t n_last = d.layers[d.n_layers - 1].N;
        struct Range { uint64_t off, len; };
        const Range r[5] = {{d.x_off, (uint64_t)d.M * d.layers[0].K * 2},
                            {d.labels_off, (uint64_t)d.M * 4},
                            {d.logits_off, (uint64_t)d.M * n_last * 4},
                            {d.loss_off, 4},
                            {d.work_off, salus_train_work_bytes(d.M, d.layers, d.n_layers)}};
        for (int a = 0; a < 5; ++a) {
            if (r[a].off % 16 || r[a].off > lane_size || r[a].len > lane_size - r[a].off)
                return set_error(pool, SALUS_EINVAL, "buffer outside the job's lane");
            for (int b = 0; b < a; ++b)
                if (overlap(r[a].off, r[a].len, r[b].off, r[b].len))
                    return set_error(pool, SALUS_EINVAL, "lane buffers overlap");
        }
        Resolved &R = res[i];
        R.persist = base + j->off;
        R.lane = base + lane_off;
        R.h_off.push_back(d.x_off);
        uint64_t at = d.work_off, max_n = 0;
        for (uint32_t l = 0; l < d.n_layers; ++l) {
            if (l + 1 < d.n_layers) {
                R.h_off.push_back(at);
                at += up256((uint64_t)d.M * d.layers[l].N * 2);
            }
            max_n = std::max<uint64_t>(max_n, d.layers[l].N);
        }
        for (uint32_t b = 0; b < std::max<uint32_t>(d.n_layers, 2); ++b)
            R.g_off.push_back(at + b * up256((uint64_t)d.M * max_n * 2));
        depth = std::max(depth, d.n_layers);
    }
    hipError_t e = hipSuccess;
    uint64_t *count = &pool->gemm_launches;
    // forward, one launch per layer depth
    std::vector<Problem> probs;
    for (uint32_t l = 0; l < depth && e == hipSuccess; ++l) {
        probs.clear();
        for (uint32_t i = 0; i < n; ++i) {
            const salus_train_desc &d = descs[i];
            if (l >= d.n_layers) continue;
            const bool last = l + 1 == d.n_layers;
            Problem pr{};
            pr.W = res[i].persist + d.layers[l].wb_off;
            pr.X = res[i].lane + res[i].h_off[l];
            pr.Y = last ? res[i].lane + d.logits_off : res[i].lane + res[i].h_off[l + 1];
            pr.M = d.M;
            pr.K = d.layers[l].K;
            pr.N = d.layers[l].N;
            pr.flags = last ? (uint32_t)SALUS_ACT_NONE : ((uint32_t)SALUS_ACT_RELU | kOutBf16);
            probs.push_back(pr);
        }
        e = launch_grouped_bf16(probs.data(), (uint32_t)probs.size(), false, stream, count);
    }
    // loss and its gradient
    if (e == hipSuccess) {
        std::vector<LossProblem> lp;
        for (uint32_t i = 0; i < n; ++i) {
            const salus_train_desc &d = descs[i];
            LossProblem p{};
            p.logits = (const float *)(res[i].lane + d.logits_off);
            p.labels = (const int32_t *)(res[i].lane + d.labels_off);
            p.grad = res[i].lane + res[i].g_off[0];
            p.loss = (float *)(res[i].lane + d.loss_off);
            p.row_loss = (float *)(res[i].lane + res[i].g_off[1]);   // a gradient buffer that is idle here
            p.M = d.M;
            p.N = d.layers[d.n_layers - 1].N;
            lp.push_back(p);
        }
        e = launch_softmax_xent(lp.data(), (uint32_t)lp.size(), stream, count);
    }
    // backward: layer `back` counted from each job's last layer, so that jobs of
    // different depth still share launches.  First the chain of input gradients
    // (step `back` reads gradient buffer `back`, writes `back + 1`), then ONE launch
    // that updates every layer of every job: the updates overwrite weights the input
    // gradients read, and one grid of all layers ramps up and drains once instead
    // of once per layer.  (Measured slower, so not done: the update of a layer on a
    // second stream, or in the same launch, beside the next input gradient - under
    // the update's HBM stream the latency-bound input gradient takes 3 - 4 times as
    // long as alone and the launch waits for it.)
    std::vector<UpdateProblem> ups;
    for (uint32_t back = 0; back < depth && e == hipSuccess; ++back) {
        probs.clear();
        for (uint32_t i = 0; i < n; ++i) {
            const salus_train_desc &d = descs[i];
            if (back >= d.n_layers) continue;
            const uint32_t l = d.n_layers - 1 - back;
            const salus_train_layer &L = d.layers[l];
            char *g_cur = res[i].lane + res[i].g_off[back];
            if (l > 0) {
                Problem pr{};
                pr.W = res[i].persist + L.wb_off;      // K x N: rows are the output columns of dX
                pr.X = g_cur;
                pr.Y = res[i].lane + res[i].g_off[back + 1];
                pr.aux = res[i].lane + res[i].h_off[l];
                pr.M = d.M;
                pr.K = L.N;
                pr.N = L.K;
                pr.flags = kOutBf16 | kMaskPositive;
                probs.push_back(pr);
            }
            UpdateProblem up{};
            up.H = res[i].lane + res[i].h_off[l];
            up.G = g_cur;
            up.Wm = (float *)(res[i].persist + L.wm_off);
            up.Wb = res[i].persist + L.wb_off;
            up.M = d.M;
            up.K = L.K;
            up.N = L.N;
            up.lr = d.lr;
            ups.push_back(up);
        }
        if (!probs.empty()) e = launch_grouped_bf16(probs.data(), (uint32_t)probs.size(), true, stream, count);
    }
    if (e == hipSuccess) e = launch_grouped_dw_sgd(ups.data(), (uint32_t)ups.size(), stream, count);
    if (e != hipSuccess) return set_error(pool, SALUS_EHIP, hipGetErrorString(e));
    return SALUS_OK;
}

int32_t salus_switch_out(salus_pool_t *pool, int32_t job, void *pinned_or_null)
{
    CHECK_POOL(pool);
    return done(pool, pool->core->switch_out(job, pinned_or_null));
}

int32_t salus_switch_in(salus_pool_t *pool, int32_t job)
{
    CHECK_POOL(pool);
    return done(pool, pool->core->switch_in(job));
}

// Starts host <-> device traffic for a held job on the caller's copy stream,
// ordered after everything already submitted to the pool's stream.
static int32_t start_transfer(salus_pool *pool, int32_t job, void *host, uint64_t off, uint64_t len,
                              bool to_host, hipStream_t copy_stream)
{
    HipOps &ops = pool->ops;
    if (!ops.present()) return SALUS_OK;
    HipOps::Transfer t{};
    hipError_t e = hipEventCreateWithFlags(&t.fence, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&t.done, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventRecord(t.fence, ops.stream);
    if (e == hipSuccess) e = hipStreamWaitEvent(copy_stream, t.fence, 0);
    if (e == hipSuccess && len)
        e = to_host ? hipMemcpyAsync(host, ops.base + off, len, hipMemcpyDeviceToHost, copy_stream)
                    : hipMemcpyAsync(ops.base + off, host, len, hipMemcpyHostToDevice, copy_stream);
    if (e == hipSuccess) e = hipEventRecord(t.done, copy_stream);
    t.failed = e != hipSuccess;
    ops.inflight[job] = t;      // also on failure: the events are released when the job is freed
    if (e != hipSuccess) return set_error(pool, SALUS_EHIP, std::string("transfer: ") + hipGetErrorString(e));
    return SALUS_OK;
}

// SALUS_OK when the job's transfer has completed (events released), SALUS_EBUSY
// when it has not and wait == 0.
static int32_t finish_transfer(salus_pool *pool, int32_t job, int32_t wait)
{
    HipOps &ops = pool->ops;
    auto it = ops.inflight.find(job);
    if (it == ops.inflight.end()) return SALUS_OK;
    if (it->second.failed)
        return set_error(pool, SALUS_EHIP, "the job's transfer failed; its bytes are not where they "
                                           "should be: free the job with salus_lane_free");
    hipError_t e = wait ? hipEventSynchronize(it->second.done) : hipEventQuery(it->second.done);
    if (e == hipErrorNotReady) return set_error(pool, SALUS_EBUSY, "transfer still in flight");
    if (e != hipSuccess) {
        // the job stays held and the failure is remembered: a second call must not
        // find "nothing in flight" and complete the bookkeeping of a copy that never landed
        it->second.failed = true;
        return set_error(pool, SALUS_EHIP, std::string("transfer: ") + hipGetErrorString(e));
    }
    (void)hipEventDestroy(it->second.fence);
    (void)hipEventDestroy(it->second.done);
    ops.inflight.erase(it);
    return SALUS_OK;
}

int32_t salus_switch_out_begin(salus_pool_t *pool, int32_t job, void *pinned_or_null, void *copy_stream)
{
    CHECK_POOL(pool);
    void *host = nullptr;
    uint64_t off = 0, len = 0;
    if (int32_t rc = pool->core->begin_out(job, pinned_or_null, &host, &off, &len)) return done(pool, rc);
    return start_transfer(pool, job, host, off, len, true, (hipStream_t)copy_stream);
}

int32_t salus_switch_out_end(salus_pool_t *pool, int32_t job, int32_t wait)
{
    CHECK_POOL(pool);
    const Job *j = pool->core->job(job);
    if (!j || !j->held || !j->leaving)
        return set_error(pool, SALUS_EINVAL, "no device-to-host transfer was begun for this job");
    if (int32_t rc = finish_transfer(pool, job, wait)) return rc;
    return done(pool, pool->core->end_out(job));
}

int32_t salus_switch_in_begin(salus_pool_t *pool, int32_t job, void *copy_stream)
{
    CHECK_POOL(pool);
    void *host = nullptr;
    uint64_t off = 0, len = 0;
    if (int32_t rc = pool->core->begin_in(job, &host, &off, &len)) return done(pool, rc);
    return start_transfer(pool, job, host, off, len, false, (hipStream_t)copy_stream);
}

int32_t salus_switch_in_end(salus_pool_t *pool, int32_t job, int32_t wait)
{
    CHECK_POOL(pool);
    const Job *j = pool->core->job(job);
    if (!j || !j->held || j->leaving)
        return set_error(pool, SALUS_EINVAL, "no host-to-device transfer was begun for this job");
    if (int32_t rc = finish_transfer(pool, job, wait)) return rc;
    return done(pool, pool->core->end_in(job));
}

int32_t salus_compact(salus_pool_t *pool, salus_move *plan_out, uint32_t cap, uint32_t *n_moves)
{
    CHECK_POOL(pool);
    std::vector<salus_move> plan;
    int32_t rc = pool->core->compact(&plan);
    if (n_moves) *n_moves = (uint32_t)plan.size();
    if (plan_out)
        for (uint32_t i = 0; i < cap && i < plan.size(); ++i) plan_out[i] = plan[i];
    return done(pool, rc);
}

int32_t salus_get_stats(salus_pool_t *pool, salus_stats *out)
{
    CHECK_POOL(pool);
    if (!out) return SALUS_EINVAL;
    *out = pool->core->stats;
    out->gemm_launches = pool->gemm_launches;
    out->fused_timeouts = pool->fused_timeouts;
    out->queued = pool->core->queued();
    return SALUS_OK;
}

int32_t salus_poll_events(salus_pool_t *pool, salus_event *out, uint32_t cap, uint32_t *n)
{
    CHECK_POOL(pool);
    if (!n) return SALUS_EINVAL;
    std::vector<salus_event> &ev = pool->core->events;
    uint32_t k = (uint32_t)std::min<size_t>(cap, ev.size());
    if (!out) k = 0;
    for (uint32_t i = 0; i < k; ++i) out[i] = ev[i];
    ev.erase(ev.begin(), ev.begin() + k);
    *n = k;
    return SALUS_OK;
}

int32_t salus_lanes(salus_pool_t *pool, int32_t *ids, uint64_t *offs, uint64_t *sizes, uint32_t cap,
                    uint32_t *n)
{
    CHECK_POOL(pool);
    if (!n) return SALUS_EINVAL;
    const std::vector<Lane> &lanes = pool->core->lanes();
    uint64_t top = pool->core->capacity();
    uint32_t k = 0;
    for (const Lane &l : lanes) {
        top -= l.bytes();
        if (k < cap) {
            if (ids) ids[k] = l.id;
            if (offs) offs[k] = top;
            if (sizes) sizes[k] = l.bytes();
            ++k;
        }
    }
    *n = (uint32_t)lanes.size();
    return SALUS_OK;
}

const char *salus_last_error(salus_pool_t *pool) { return pool ? pool->error.c_str() : "null pool"; }

// ---- device self-checks ------------------------------------------------------
int32_t salus_scan_u64(const uint64_t *host_in, uint32_t n, uint64_t *host_out, void *scratch,
                       void *stream)
{
    if (!host_in || !host_out || !scratch || n > 4096) return SALUS_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    uint64_t *in = (uint64_t *)scratch, *out = in + n;
    hipError_t e = hipMemcpyAsync(in, host_in, (size_t)n * 8, hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = launch_scan_u64(in, n, out, s);
    if (e == hipSuccess) e = hipMemcpyAsync(host_out, out, ((size_t)n + 1) * 8, hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    return e == hipSuccess ? SALUS_OK : SALUS_EHIP;
}

int32_t salus_fill_pattern(void *dev, uint64_t nbytes, uint64_t seed, void *stream)
{
    if (!dev || nbytes % 8 || (uintptr_t)dev % 8) return SALUS_EINVAL;
    hipError_t e = launch_fill_pattern(dev, nbytes, seed, (hipStream_t)stream);
    if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);
    return e == hipSuccess ? SALUS_OK : SALUS_EHIP;
}

int32_t salus_check_pattern(const void *dev, uint64_t nbytes, uint64_t seed, void *scratch,
                            uint64_t *bad, void *stream)
{
    if (!dev || !scratch || !bad || nbytes % 8 || (uintptr_t)dev % 8) return SALUS_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    unsigned long long zero = 0, got = 0;
    hipError_t e = hipMemcpyAsync(scratch, &zero, 8, hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = launch_check_pattern(dev, nbytes, seed, (unsigned long long *)scratch, s);
    if (e == hipSuccess) e = hipMemcpyAsync(&got, scratch, 8, hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    *bad = got;
    return e == hipSuccess ? SALUS_OK : SALUS_EHIP;
}

int32_t salus_pack_strip128(const uint16_t *src, uint16_t *dst, uint32_t K, uint32_t N)
{
    if (!src || !dst || N % 128) return SALUS_EINVAL;
    for (uint32_t s = 0; s < N / 128; ++s)
        for (uint32_t k = 0; k < K; ++k)
            std::memcpy(dst + ((size_t)s * K + k) * 128, src + (size_t)k * N + (size_t)s * 128, 256);
    return SALUS_OK;
}

int32_t salus_calibrate_read(const void *dev, uint64_t nbytes, void *dev_sink, void *stream)
{
    if (!dev || !dev_sink || nbytes % 4096 || (uintptr_t)dev % 16 || (uintptr_t)dev_sink % 16) return SALUS_EINVAL;
    return launch_read_only(dev, nbytes, dev_sink, (hipStream_t)stream) == hipSuccess ? SALUS_OK : SALUS_EHIP;
}

int32_t salus_calibrate_mfma(void *dev_out, uint32_t slabs, int32_t from_lds, void *stream, uint64_t *flop)
{
    if (!dev_out || !slabs || (uintptr_t)dev_out % 8) return SALUS_EINVAL;
    return launch_mfma_rate((uint64_t *)dev_out, slabs, from_lds != 0, (hipStream_t)stream, flop) == hipSuccess
               ? SALUS_OK : SALUS_EHIP;
}

int32_t salus_copy(void *dst, const void *src, uint64_t nbytes, void *stream)
{
    if (!dst || !src || nbytes % 16 || (uintptr_t)dst % 16 || (uintptr_t)src % 16) return SALUS_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    hipError_t e;
    const char *sp = (const char *)src;
    char *dp = (char *)dst;
    if (dp + nbytes <= sp || sp + nbytes <= dp) {
        CopySeg seg{src, dst, nbytes};
        e = launch_copy(&seg, 1, s);
    } else if (dp < sp) {
        // this self-check has no pool: its in-place moves share one set of counters per device
        // (kept until the process ends), so overlapping calls of salus_copy must not run concurrently
        static SlideState states[kMaxDevices];
        int dev = -1;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SALUS_EHIP;
        SlideState &state = states[dev];
        if (!state.progress && slide_state_create(&state) != hipSuccess) return SALUS_EHIP;
        uint64_t so = (uint64_t)(sp - dp), zo = 0, len = nbytes;   // offsets relative to dst
        e = launch_slide(dp, &so, &zo, &len, 1, &state, s, nullptr);
        uint32_t gave_up = 0;
        if (e == hipSuccess) e = slide_state_failed(&state, s, &gave_up);
        if (e == hipSuccess && gave_up) return SALUS_ETIMEOUT;
    } else {
        return SALUS_EINVAL;    // moving upward with overlap is never needed by the pool
    }
    return e == hipSuccess ? SALUS_OK : SALUS_EHIP;
}

}  // extern "C"
