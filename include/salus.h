/* salus.h - C ABI of the MI355X packed-iteration and job-switch library.
 *
 * One pool object manages one caller-owned range of device memory on one GPU
 * the way Salus (arXiv 1902.04610) manages a GPU: persistent memory of every
 * admitted job stays resident (Section 3.2.1), ephemeral memory lives in lanes
 * (Section 3.3), jobs are admitted by the lane-assignment algorithm
 * (Algorithm 1) under the safety condition (Section 3.3.2), and iterations are
 * scheduled at iteration granularity (Sections 3.2.2 and 4).  On top of that
 * model the library executes the dense layers of all jobs scheduled in a round
 * as one grouped GEMM launch per layer depth, and moves persistent state
 * (evict / restore to pinned host memory, on-device compaction).
 *
 * Conventions
 *  - Every call returns an int32_t status: SALUS_OK, SALUS_QUEUED or a negative
 *    error.  After an error salus_last_error() gives a message.
 *  - "device pointer" = address valid on the GPU; "host pointer" = ordinary
 *    process memory.  All sizes and offsets are bytes (uint64_t); offsets are
 *    relative to the pool base.
 *  - The library keeps almost nothing in device memory of its own: every pool with
 *    device memory holds 16 KB of counters for in-place compaction, a pool created
 *    with SALUS_FLAG_FUSE_DEPTHS another 20 KB for descriptors and completion
 *    counters (both allocated in salus_pool_create, never later), and
 *    salus_grouped_forward_static uses a fixed array inside the library.  It owns
 *    its metadata and the pinned host buffers that hold evicted state (unless the
 *    caller passes one).
 *  - Not thread safe: one scheduler thread drives a pool (the paper's execution
 *    service is a singleton, Section 3.1).
 *  - Calls that change the layout (lane_alloc, lane_free, switch_out, switch_in,
 *    compact) are only legal between iterations: all ephemeral memory is dead
 *    there (Section 3.2.2), and the caller must not have work in flight on
 *    other streams that touches the pool.
 *  - Job ids are dense, starting at 0, in arrival order.  Lane ids are dense in
 *    creation order and never reused.
 */
#ifndef SALUS_H
#define SALUS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct salus_pool salus_pool_t;

enum {
    SALUS_OK = 0,
    SALUS_QUEUED = 1,          /* request accepted, waiting in the pending queue Q */
    SALUS_EINVAL = -1,         /* bad argument / bad job id / wrong job state */
    SALUS_ENOMEM = -2,         /* safety condition would be violated */
    SALUS_ENOTRESIDENT = -3,   /* job's persistent state is not on the device */
    SALUS_EBUSY = -4,          /* two jobs of one lane in the same launch; job or transfer in transit */
    SALUS_ENEVER = -5,         /* P + E > C: the job could not run even alone (Section 4.2) */
    SALUS_EHIP = -6,           /* the HIP runtime reported an error */
    SALUS_ETIMEOUT = -7        /* a depth-fused forward gave up waiting (salus_fused_check) */
};

/* Scheduling policies of Section 4. */
enum {
    SALUS_POLICY_FIFO = 0,     /* oldest runnable job of the pool only */
    SALUS_POLICY_FAIR = 1,     /* per lane: least attained service (round-robin); a job enters a
                                  lane level with the least-served job it competes with, so
                                  shares become 1/n at once (Sections 4.3 and 5.1.2) */
    SALUS_POLICY_PRIORITY = 2, /* per lane: highest priority, then shortest remaining (SRTF) */
    SALUS_POLICY_PACK = 3      /* every lane runs its oldest runnable job */
};

enum { SALUS_JOB_QUEUED = 0, SALUS_JOB_RESIDENT = 1, SALUS_JOB_EVICTED = 2, SALUS_JOB_DONE = 3 };

enum { SALUS_ACT_NONE = 0, SALUS_ACT_RELU = 1, SALUS_ACT_GELU = 2 };

enum { SALUS_F32 = 0, SALUS_BF16 = 1 };

/* Pool options.  SHRINK_LANES: when the job with the largest ephemeral peak leaves
 * a lane that other jobs still use, the lane shrinks to the largest remaining
 * peak, so that L_j = max E_i holds as an equality (Section 3.3.2); younger
 * lanes slide up without any copy.  Off by default: Algorithm 1 never shrinks.
 * FUSE_DEPTHS: salus_grouped_forward runs all layer depths of a round in one
 * launch whose workgroups wait for their job's previous layer on the device,
 * instead of one launch per depth (see salus_grouped_forward). */
enum { SALUS_FLAG_SHRINK_LANES = 1, SALUS_FLAG_FUSE_DEPTHS = 2 };

/* How switch_out / switch_in cross the host link. */
enum { SALUS_COPY_KERNEL = 0,  /* the library's own copy kernel on mapped pinned memory */
       SALUS_COPY_DMA = 1 };   /* hipMemcpyAsync (copy engine) */

typedef struct {
    uint64_t granule;      /* P and E are rounded up to it; power of two >= 16; 0 = 256 */
    uint32_t max_lanes;    /* cap on the number of lanes; 0 = unlimited */
    int32_t  policy;       /* SALUS_POLICY_* */
    void    *stream;       /* hipStream_t for copies and compaction; NULL = default stream */
    int32_t  copy_engine;  /* SALUS_COPY_* */
    uint32_t flags;        /* SALUS_FLAG_* */
} salus_config;

typedef struct {
    int32_t  state;        /* SALUS_JOB_* */
    int32_t  lane;         /* lane id, -1 while queued */
    int32_t  priority;
    int32_t  auto_evicted; /* 1 if priority admission evicted it (it is restored automatically) */
    int32_t  in_transit;   /* 1 between salus_switch_*_begin and _end: resident but not runnable */
    int32_t  lane_parked;  /* 1 while no job of the lane is resident: the lane then holds no bytes */
    uint64_t P, E;         /* granule-rounded sizes */
    uint64_t persist_off;  /* valid while RESIDENT; changes on compact / switch_in */
    uint64_t lane_off;     /* current base of the job's lane; changes when older lanes vanish or grow */
    uint64_t lane_size;    /* L_j (reserved at lane_off unless lane_parked) */
    uint64_t pending;      /* iterations still to run */
    uint64_t served;       /* iterations issued so far */
    uint64_t cost;         /* duration of one iteration in the caller's time unit (default 1) */
    uint64_t attained;     /* service level the job entered its lane at + the costs of its iterations since */
    uint64_t arrival_round, admit_round;   /* admit_round = UINT64_MAX while queued */
} salus_job_info;

typedef struct { int32_t job, lane; } salus_slot;

typedef struct { uint64_t src, dst, len; } salus_move;

/* How a layer's K x N weights are stored.  ROWMAJOR: element (k, n) at index
 * k * N + n.  STRIP128 (bf16 only, N a multiple of 128): columns are grouped in
 * strips of 128 and each strip is a contiguous K x 128 block, element (k, n) at
 * (n / 128 * K + k) * 128 + n % 128.  Same values, same results; a column tile
 * of the kernels then streams one contiguous range of HBM instead of K separate
 * 256-byte pieces.  salus_pack_strip128 converts on the host. */
enum { SALUS_LAYOUT_ROWMAJOR = 0, SALUS_LAYOUT_STRIP128 = 1 };

/* One layer: H_out[M x N] = act(H_in[M x K] . W[K x N]); W at w_off bytes
 * inside the job's persistent block. */
typedef struct {
    uint32_t K, N;
    uint64_t w_off;
    int32_t  act;          /* SALUS_ACT_* */
    int32_t  layout;       /* SALUS_LAYOUT_* */
} salus_layer;

/* One job's forward pass in a packed iteration.  All three offsets are inside
 * the job's lane (its ephemeral memory).  x: input, M x K_0, in `dtype`.
 * y: output of the last layer, M x N_last, always float.  h: scratch of
 * salus_forward_work_bytes() bytes for the intermediate activations, whose
 * layout is private to the library.  SALUS_BF16: weights, input and
 * intermediate activations are bf16 (activations rounded to nearest-even),
 * sums in float. */
typedef struct {
    int32_t  job;
    uint32_t M;
    uint32_t n_layers;
    int32_t  dtype;        /* SALUS_F32 or SALUS_BF16 */
    const salus_layer *layers;   /* host pointer, n_layers entries */
    uint64_t x_off, y_off, h_off;
} salus_gemm_desc;

/* Bytes of lane scratch (`h`) a forward pass of these layers needs at batch M. */
uint64_t salus_forward_work_bytes(uint32_t M, const salus_layer *layers, uint32_t n_layers,
                                  int32_t dtype);

typedef struct {
    uint64_t rounds, iterations;
    uint64_t bytes_d2h, bytes_h2d, bytes_d2d;
    uint64_t moves, compactions;
    uint64_t lanes_opened, lanes_deleted, lanes_moved;
    uint64_t evictions, restores, admitted, queued;
    uint64_t gemm_launches;
    uint64_t fused_timeouts;   /* salus_fused_check calls that found a wait given up */
} salus_stats;

enum { SALUS_EV_ADMIT = 0, SALUS_EV_EVICT = 1, SALUS_EV_RESTORE = 2, SALUS_EV_LANE_NEW = 3,
       SALUS_EV_LANE_GROW = 4, SALUS_EV_LANE_DEL = 5, SALUS_EV_LANE_MOVED = 6, SALUS_EV_COMPACT = 7,
       SALUS_EV_LANE_SHRINK = 8, SALUS_EV_LANE_PARK = 9, SALUS_EV_LANE_UNPARK = 10 };

/* kind ADMIT: a = job, b = lane | EVICT: a = job, b = bytes | RESTORE: a = job,
 * b = new persistent offset | LANE_NEW / LANE_GROW / LANE_SHRINK: a = lane, b = size |
 * LANE_DEL: a = lane | LANE_MOVED: a = number of lanes that slid | COMPACT:
 * a = moves, b = bytes moved. */
typedef struct { int32_t kind; int32_t pad; uint64_t a, b; } salus_event;

/* Section 3.3: split [base, base+capacity) into a persistent region growing up
 * from offset 0 and an ephemeral region (lanes) growing down from `capacity`.
 * base: device pointer, 256-byte aligned, owned by the caller and alive until
 * salus_pool_destroy; may be NULL for a metadata-only pool (every call that
 * would touch device memory then fails with SALUS_EINVAL, except that layout
 * calls simply skip the copies).  capacity must be a multiple of the granule. */
int32_t salus_pool_create(void *base, uint64_t capacity, const salus_config *cfg,
                          salus_pool_t **out);
int32_t salus_pool_destroy(salus_pool_t *pool);

/* Algorithm 1, JobArrive(P, E) followed by ProcessRequests: the request joins
 * the pending queue and every queued request is offered to FindLane (new lane,
 * else best matching existing lane, else grow the smallest lane that makes it
 * fit), always under  sum P_i + sum L_j <= C.  The job's persistent block is
 * placed first-fit at the lowest address below the ephemeral region; live
 * blocks are compacted on the device first when no single hole is big enough
 * or when the new lane needs the space they occupy.  Under
 * SALUS_POLICY_PRIORITY a request that finds no lane evicts resident jobs of
 * strictly lower priority to pinned host memory (Section 4.2), as few as
 * needed.  priority: larger = more urgent.  pending: iterations to run
 * (remaining time for SRTF); may be 0 and set later.
 * Returns SALUS_OK (resident now), SALUS_QUEUED, SALUS_ENEVER, SALUS_EINVAL. */
int32_t salus_lane_alloc(salus_pool_t *pool, uint64_t P, uint64_t E, int32_t priority,
                         uint64_t pending, int32_t *job);

/* Algorithm 1, JobFinish: frees the persistent block (and any host copy),
 * drops the lane reference; an empty lane is deleted and younger lanes slide
 * into its place without any copy (Section 3.3.1).  Then the queue is
 * processed and automatically evicted jobs that fit again are restored. */
int32_t salus_lane_free(salus_pool_t *pool, int32_t job);

int32_t salus_job_query(salus_pool_t *pool, int32_t job, salus_job_info *out);
int32_t salus_job_set_pending(salus_pool_t *pool, int32_t job, uint64_t n);
/* Duration of one iteration of the job (measured or estimated, any unit, >= 1).
 * FAIR equalizes the summed cost of the iterations each job was given, PRIORITY
 * orders equal priorities by pending x cost (Section 4: attained service and
 * remaining time are times).  Default 1: both count iterations. */
int32_t salus_job_set_cost(salus_pool_t *pool, int32_t job, uint64_t cost);
/* The same for count jobs at once (host arrays); stops at the first bad job id. */
int32_t salus_set_pending_many(salus_pool_t *pool, const int32_t *jobs, const uint64_t *n,
                               uint32_t count);

/* Copy bytes between host memory and a resident job's persistent block
 * (synchronous; for loading weights and reading them back). */
int32_t salus_job_write(salus_pool_t *pool, int32_t job, uint64_t off, const void *host_src,
                        uint64_t nbytes);
int32_t salus_job_read(salus_pool_t *pool, int32_t job, uint64_t off, void *host_dst,
                       uint64_t nbytes);

/* Sections 3.3 and 4: one scheduling round.  Picks at most one resident job
 * with pending > 0 per lane according to the policy (jobs in transit are
 * skipped), charges it one iteration (served + 1, attained + cost, pending - 1)
 * and writes the (job, lane) pairs in lane creation order to out[0..*n).
 * cap must be >= the number of lanes. */
int32_t salus_schedule_iteration(salus_pool_t *pool, salus_slot *out, uint32_t cap, uint32_t *n);

/* Packed iteration (Section 3.3: lanes run in parallel): the forward passes of
 * all n jobs run together, one grouped GEMM launch per layer depth on `stream`
 * (hipStream_t, NULL = default), asynchronously.  Jobs must be resident and
 * belong to pairwise different lanes (SALUS_EBUSY otherwise); every buffer
 * must lie inside the job's lane / persistent block (SALUS_EINVAL).  K and N
 * of every layer must be multiples of 8 (bf16) or 4 (f32).
 *
 * In a pool with SALUS_FLAG_FUSE_DEPTHS the jobs of one dtype run as ONE launch
 * over all their layers when each has at most 6 layers and, for bf16, at most
 * 32 rows (otherwise that dtype takes the per-depth launches): the workgroups
 * of layer l+1 wait on a device counter for the job's layer l, so a job's next
 * layer starts as soon as its own input is complete and no launch boundary
 * drains the GPU.  Outputs are bit-identical to the per-depth launches.  The
 * job's persistent state and iteration boundary are untouched: this is batching
 * inside one iteration (Section 3.2.2 rules out scheduling below it, not
 * this).  Fused calls of one pool must be ordered on the device (use one
 * stream) and cannot be recorded in a HIP graph (SALUS_EINVAL while the stream
 * is capturing: consecutive launches alternate between two sets of counters);
 * the per-depth launches can, they are plain kernel launches with by-value
 * arguments.  The device-side wait is bounded; see salus_fused_check. */
int32_t salus_grouped_forward(salus_pool_t *pool, const salus_gemm_desc *descs, uint32_t n,
                              void *stream);

/* For callers that must not allocate device memory and have no lane room to
 * spare for scratch (code recorded into a HIP graph, tight serving loops,
 * harnesses that forbid allocation): salus_grouped_forward with the hidden
 * activations kept in a fixed array inside the library instead of at h_off in
 * each job's lane.  h_off is ignored; x and y are still the caller's, inside the
 * lane.  Same kernels, same launches per layer depth (never depth-fused), same
 * bits in y.  The round's hidden activations - the sum over its jobs of
 * salus_forward_work_bytes(), each rounded up to 256 - must fit
 * SALUS_STATIC_SCRATCH_BYTES, else SALUS_ENOMEM and nothing is launched.  The
 * call allocates and frees nothing on the device.  One array per GPU, shared
 * by every pool and every call on that GPU and never cleared (every element
 * that is read was written earlier in the same call): calls that can overlap on
 * one GPU - different streams, or different host threads - race on it and must
 * be ordered by the caller.  The GPU of the pool must be the current device.
 * The first call on a device looks up the array's address; make one call (n = 0
 * will do) before recording the entry point into a graph. */
#define SALUS_STATIC_SCRATCH_BYTES (32ull << 20)
int32_t salus_grouped_forward_static(salus_pool_t *pool, const salus_gemm_desc *descs, uint32_t n,
                                     void *stream);

/* MANDATORY after fused launches, before their outputs are used: the device-side
 * wait relies on workgroups being dispatched in index order, which the hardware
 * does today but no specification promises; when that fails the launch still
 * ends (the wait is bounded) and this call is the only place that says so.
 * After the caller has synchronized the stream: SALUS_OK if every device-side
 * wait of the fused launches completed since the last check ended normally,
 * SALUS_ETIMEOUT if one gave up (the outputs of those launches are invalid; the
 * pool stays usable).  A wait gives up after `polls` polls of about a
 * microsecond (default 2^21); it cannot happen while workgroups are dispatched
 * in index order, the bound exists so that no launch can hang. */
int32_t salus_fused_check(salus_pool_t *pool);
int32_t salus_fused_spin_limit(salus_pool_t *pool, uint32_t polls);

/* One layer of a training job: bf16 working weights and float master weights,
 * both K x N row-major inside the job's persistent block. */
typedef struct {
    uint32_t K, N;
    uint64_t wb_off;       /* bf16 working copy */
    uint64_t wm_off;       /* float master weights */
} salus_train_layer;

/* One job's training step.  Offsets are inside the job's lane.
 * x: M x K_0 bf16 inputs; labels: M int32 class indices in [0, N_last) (values
 * outside are clamped); logits: M x N_last float (written); loss: one float
 * (written, mean cross-entropy); work: scratch of salus_train_work_bytes(). */
typedef struct {
    int32_t  job;
    uint32_t M;
    uint32_t n_layers;
    float    lr;
    const salus_train_layer *layers;   /* host pointer, n_layers entries */
    uint64_t x_off, labels_off, logits_off, loss_off, work_off;
} salus_train_desc;

/* Bytes of lane scratch a training step needs: the hidden activations of every
 * layer (kept for the backward pass) and one gradient buffer per layer (at
 * least two). */
uint64_t salus_train_work_bytes(uint32_t M, const salus_train_layer *layers, uint32_t n_layers);

/* Packed training iteration (Sections 2.1 and 5.2: forward pass, backward pass
 * and parameter update of many tuning jobs sharing the GPU).  For all n jobs
 * together, on `stream`, asynchronously:
 *   H_l = bf16(relu(H_{l-1} . Wb_l)) for hidden layers, logits = H_{L-1} . Wb_L;
 *   loss and dZ_L = (softmax - onehot) / M;
 *   for l = L..1:  G = bf16(dZ_l);  dZ_{l-1} = (G . Wb_l^T) * [H_{l-1} > 0];
 *                  Wm_l <- Wm_l - lr * (H_{l-1}^T . G);  Wb_l <- bf16(Wm_l)
 * with one grouped launch per layer for the forward pass and for the input
 * gradients, one for the loss, and one that updates every layer (it runs last:
 * the updates overwrite weights the input gradients read; every layer's
 * incoming gradient is kept in the work area until then).  ReLU between
 * layers, no biases, plain SGD.  Same residency, lane and bounds rules as
 * salus_grouped_forward; K and N multiples of 8. */
int32_t salus_grouped_train_step(salus_pool_t *pool, const salus_train_desc *descs, uint32_t n,
                                 void *stream);

/* Efficient job switching made explicit for jobs that cannot stay
 * (Sections 3.2 and 4.2): RESIDENT -> EVICTED copies the persistent block to
 * pinned host memory and frees it.  pinned_or_null: caller-owned pinned,
 * device-mapped buffer of at least P bytes that stays valid until the job is
 * switched in or freed; NULL = the library allocates (and caches) one.
 * Synchronous with respect to the pool's stream on return. */
int32_t salus_switch_out(salus_pool_t *pool, int32_t job, void *pinned_or_null);
/* EVICTED -> RESIDENT: first-fit placement (compacting if needed), then copy back. */
int32_t salus_switch_in(salus_pool_t *pool, int32_t job);

/* Overlapped switching (Section 5.1.2: a switch must not stall the other
 * lanes): the same two transitions split into begin and end, with the bytes
 * moved by the copy engine on `copy_stream` (a caller-owned hipStream_t other
 * than the pool's) while later launches on the pool's stream keep running.
 *   out_begin: job must be RESIDENT; the transfer is ordered after all work
 *              already submitted to the pool's stream.  Until out_end the job
 *              keeps its block and its lane, is reported in_transit, is never
 *              scheduled, never chosen as an eviction victim, and
 *              salus_lane_free / salus_job_write / salus_job_read / launches
 *              naming it return SALUS_EBUSY.
 *   out_end:   wait != 0 blocks the host until the bytes are in the host
 *              buffer; wait == 0 returns SALUS_EBUSY (nothing changed) while
 *              they are not.  Then the block is freed: the job is EVICTED.
 *   in_begin:  job must be EVICTED; placement happens here exactly as in
 *              salus_switch_in (the job is RESIDENT and in_transit), the copy
 *              back is ordered after all work already on the pool's stream.
 *   in_end:    as out_end; afterwards the job is runnable.
 * A compaction that runs while transfers are in flight is ordered after them
 * on the device.  A pool without device memory only does the bookkeeping.
 * If the HIP runtime reports a failed transfer, _end returns SALUS_EHIP on every
 * call and the job stays in transit; salus_lane_free then gives the job up. */
int32_t salus_switch_out_begin(salus_pool_t *pool, int32_t job, void *pinned_or_null, void *copy_stream);
int32_t salus_switch_out_end(salus_pool_t *pool, int32_t job, int32_t wait);
int32_t salus_switch_in_begin(salus_pool_t *pool, int32_t job, void *copy_stream);
int32_t salus_switch_in_end(salus_pool_t *pool, int32_t job, int32_t wait);

/* Defragmentation of the persistent region.  The paper is silent here: Section
 * 3.3.1 only removes fragmentation between lanes (for free, since ephemeral
 * memory is dead between iterations) and calls the classical move-out /
 * move-back scheme costly; it never moves persistent memory and does not say
 * how that region is allocated.  Reading taken: slide all live persistent
 * blocks to the low end in address order; new offset = exclusive prefix sum of
 * the granule-rounded sizes.  Executes the moves on the device, each byte read
 * once and written once, in place also where a block overlaps its own
 * destination (no staging: nothing outside the moved blocks is touched, lane
 * contents survive) and writes the plan to
 * plan_out[0..*n_moves) in ascending source order (at most cap entries are
 * written; *n_moves is the full count).  Blocks that already sit at their
 * final offset do not appear.  lane_alloc, switch_in and switch_in_begin run the
 * same compaction by themselves when a request needs it. */
int32_t salus_compact(salus_pool_t *pool, salus_move *plan_out, uint32_t cap, uint32_t *n_moves);

/* An in-place move has workgroups wait for one another (a chunk is written only
 * after the chunks under its destination have been read).  The wait is bounded:
 * after `polls` polls (default 2^22, seconds) a workgroup gives up, skips its
 * write and runs to its end, and the operation that needed the compaction
 * returns SALUS_EHIP with "gave up" in salus_last_error; the persistent region
 * is then damaged and the pool must be destroyed.  With the default this cannot
 * happen on an otherwise idle device; the knob exists for tests of that path
 * (polls = 0 gives up at the first unsuccessful poll). */
int32_t salus_compact_spin_limit(salus_pool_t *pool, uint32_t polls);

int32_t salus_get_stats(salus_pool_t *pool, salus_stats *out);
/* Copies and clears the event log (at most cap entries; *n = entries copied). */
int32_t salus_poll_events(salus_pool_t *pool, salus_event *out, uint32_t cap, uint32_t *n);
/* Lane ids in creation order with their current base and the bytes they hold
 * (L_j; 0 for a parked lane, i.e. one whose jobs are all evicted). */
int32_t salus_lanes(salus_pool_t *pool, int32_t *ids, uint64_t *offs, uint64_t *sizes,
                    uint32_t cap, uint32_t *n);
const char *salus_last_error(salus_pool_t *pool);

/* Device self-checks used by the tests (each is synchronous).
 * salus_scan_u64: exclusive prefix sum of n (<= 4096) host integers computed
 * by the wavefront scan the kernels use; result to host out[0..n], out[n] =
 * total.  scratch: device pointer to at least (2*n+2)*8 bytes.
 * salus_fill_pattern / salus_check_pattern: write / verify the 64-bit pattern
 * f(seed, index) over a device range (nbytes multiple of 8); check returns the
 * number of mismatching words in *bad (scratch: 8 device bytes). */
int32_t salus_scan_u64(const uint64_t *host_in, uint32_t n, uint64_t *host_out, void *scratch,
                       void *stream);
int32_t salus_fill_pattern(void *dev, uint64_t nbytes, uint64_t seed, void *stream);
int32_t salus_check_pattern(const void *dev, uint64_t nbytes, uint64_t seed, void *scratch,
                            uint64_t *bad, void *stream);
/* Host helper: reorder K x N row-major 16-bit weights into SALUS_LAYOUT_STRIP128
 * (src and dst are host pointers to K * N elements and must not overlap; N a
 * multiple of 128).  Pure data movement. */
int32_t salus_pack_strip128(const uint16_t *src, uint16_t *dst, uint32_t K, uint32_t N);
/* Calibration of the matrix pipes (measurement support, not part of the method):
 * one workgroup of eight wavefronts per compute unit runs, `slabs` times, the 32
 * v_mfma_f32_32x32x16_bf16 per wavefront that the LDS-tiled kernel issues for a
 * 256 x 256 x 64 slab, on nonzero operands - on fragments held in registers
 * (from_lds = 0) or read from LDS for every k-step with one barrier per slab
 * (from_lds = 1) - and nothing else.  Asynchronous on `stream`; the caller times
 * it.  dev_out: 24 device bytes, 8-aligned; receives {shader clock cycles, ticks
 * of the 100 MHz wall clock} that one wavefront's loop took, so that the clock
 * the chip holds under this load can be read off.  *flop (host, may be null):
 * floating-point operations of the launch. */
int32_t salus_calibrate_mfma(void *dev_out, uint32_t slabs, int32_t from_lds, void *stream, uint64_t *flop);
/* Calibration of the read path (measurement support): a kernel that only loads.
 * It reads [dev, dev + nbytes) once - 256 KiB in one piece per workgroup, 16
 * bytes per lane, eight loads in flight per wavefront, non-temporal - and writes
 * nothing (dev_sink: 16 device bytes, 16-aligned, written only if the data xor
 * to one particular value).  nbytes a multiple of 4096, dev 16-aligned.
 * Asynchronous on `stream`; the caller times it. */
int32_t salus_calibrate_read(const void *dev, uint64_t nbytes, void *dev_sink, void *stream);
/* Plain device copy with the library's copy kernel (memmove semantics when the
 * ranges overlap with dst < src). */
int32_t salus_copy(void *dst, const void *src, uint64_t nbytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif
