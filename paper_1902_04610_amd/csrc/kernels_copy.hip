// Copy, compaction, scan and pattern kernels for gfx950.
//
// These move a job's persistent state: eviction / restore across the host link
// and on-device compaction of the persistent region.  The Salus paper keeps
// persistent memory in place (Section 3.2.1) and needs no copy for lane-level
// defragmentation (Section 3.3.1); these kernels serve the cases it leaves
// open: jobs that do not fit together (Section 4.2) and fragmentation inside
// the persistent region.
//
// All kernels are bound by memory bandwidth: every thread moves 16 bytes per
// access, consecutive lanes touch consecutive addresses, a workgroup moves one
// chunk (kCopyChunk bytes) per step, and all addressing is 64-bit (pools are far
// larger than 4 GiB).
#include <algorithm>
#include <vector>

#include "device.hpp"
#include "wave.hpp"

namespace salus {

struct CopyArgs {
    uint32_t n;
    uint32_t pad;
    CopySeg seg[kMaxSeg];
};

constexpr int kCopyThreads = 256;
constexpr int kVecPerThread = kCopyChunk / (kCopyThreads * 16);

// Grid-stride over the chunks of a list of segments.  Each wavefront holds
// segment i in lane i, scans the per-segment chunk counts to get every
// segment's first chunk number, and finds the segment of a chunk with a ballot.
__global__ __launch_bounds__(kCopyThreads) void copy_segments(CopyArgs a, uint64_t total_chunks)
{
    const int lane = threadIdx.x & 63;
    const bool valid = lane < (int)a.n;
    uint64_t my_src = 0, my_dst = 0, my_len = 0;
    if (valid) {
        my_src = (uint64_t)a.seg[lane].src;
        my_dst = (uint64_t)a.seg[lane].dst;
        my_len = a.seg[lane].len;
    }
    const uint64_t my_chunks = (my_len + kCopyChunk - 1) / kCopyChunk;
    const uint64_t first_chunk = wave_excl_scan_u64(my_chunks, nullptr);

    for (uint64_t chunk = blockIdx.x; chunk < total_chunks; chunk += gridDim.x) {
        const int s = wave_find_range(first_chunk, chunk, valid);
        const uint64_t off = (chunk - __shfl((unsigned long long)first_chunk, s, 64)) * kCopyChunk;
        const uint64_t len = __shfl((unsigned long long)my_len, s, 64);
        const u32x4 *src = (const u32x4 *)(__shfl((unsigned long long)my_src, s, 64) + off);
        u32x4 *dst = (u32x4 *)(__shfl((unsigned long long)my_dst, s, 64) + off);
        const uint64_t left = len - off;
        const uint32_t nvec = (uint32_t)((left < kCopyChunk ? left : kCopyChunk) / 16);
        u32x4 v[kVecPerThread];
#pragma unroll
        for (int j = 0; j < kVecPerThread; ++j) {
            const uint32_t i = threadIdx.x + j * kCopyThreads;
            if (i < nvec) v[j] = __builtin_nontemporal_load(src + i);
        }
#pragma unroll
        for (int j = 0; j < kVecPerThread; ++j) {
            const uint32_t i = threadIdx.x + j * kCopyThreads;
            if (i < nvec) __builtin_nontemporal_store(v[j], dst + i);
        }
    }
}

static uint32_t copy_grid(uint64_t chunks)
{
    // measured on MI355X, 8 GiB copied: one workgroup per 8 KiB chunk gives the best
    // read+write rate, 6.07 TB/s (chunks of 4 / 16 / 32 KiB: 5.61 / 5.74 / 5.47; 16 KiB
    // chunks with 8 passes over a smaller grid: 5.27).  The cap keeps grid x block
    // below 2^32 threads; beyond 64 GiB per launch the workgroups loop.
    const uint64_t cap = 1u << 23;
    return (uint32_t)std::min<uint64_t>(chunks, cap);
}

hipError_t launch_copy(const CopySeg *segs, uint32_t n, hipStream_t stream)
{
    for (uint32_t at = 0; at < n; at += kMaxSeg) {
        CopyArgs a{};
        a.n = std::min(kMaxSeg, n - at);
        uint64_t chunks = 0;
        for (uint32_t i = 0; i < a.n; ++i) {
            a.seg[i] = segs[at + i];
            chunks += (a.seg[i].len + kCopyChunk - 1) / kCopyChunk;
        }
        if (chunks == 0) continue;
        hipLaunchKernelGGL(copy_segments, dim3(copy_grid(chunks)), dim3(kCopyThreads), 0, stream, a,
                           chunks);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// ---------------------------------------------------------------------------
// In-place move toward lower addresses of a range that overlaps its own
// destination (shift = src - dst < len): the hard case of sliding compaction.
// Every byte is read once and written once, whatever the shift.
//
// The range is cut into chunks of kSlideChunk bytes, processed in ascending order
// by a grid of G workgroups that all fit on the device at once (workgroup w takes
// chunks w, w + G, ...).  A
// workgroup loads its whole chunk into registers, publishes "chunk read", and
// only then may write it.  The destination of chunk i covers source bytes of
// chunks i - q - 1 and i - q (q = shift / chunk) and of no later chunk, so the
// write has to wait until those two chunks have been read - by other workgroups,
// which need nothing from anyone to get that far.  No data passes between
// workgroups through memory, only the fact that a load has completed, so no
// cache maintenance is needed: a relaxed device-scope counter per workgroup
// (chunks read so far) is enough.
//
// Why every wait ends: G is at most two workgroups per compute unit of a kernel
// that fits at least that many (checked with the occupancy query), so the grid
// fits the device by itself; workgroups of other kernels that happen to run end
// on their own, so all G workgroups become resident, and from then on the lowest
// unwritten chunk never waits for anything that is not already under way.  (A
// cooperative launch would have the runtime check the same fit; it is not used
// because the profiler of this ROCm release crashes at exit after one.)  The wait
// is bounded all the same; a workgroup that gives up sets `*failed`, skips its
// write and carries on publishing its reads, so that every wavefront exits.  The
// host then reports the compaction as failed.
// ---------------------------------------------------------------------------
// measured on MI355X, 8 GB moved down by 256 B / 48 KiB / 40 MiB (read + write): chunks of 32 KiB 5.3 / 5.2 / 5.3 TB/s,
// 64 KiB 5.5 / 5.5 / 5.3, 128 KiB 5.7 / 5.7 / 5.4, 192 KiB 5.9 / 5.9 / 5.8, 256 KiB 5.9 / 5.9 / 5.5 (192 KiB is
// 192 registers per lane, two workgroups per compute unit); more workgroups per compute unit: no difference
constexpr uint32_t kSlideChunk = 192 * 1024;
constexpr int kSlideVec = kSlideChunk / (kCopyThreads * 16);

__global__ void slide_reset(uint32_t *progress, uint32_t n, uint32_t *failed)
{
    for (uint32_t i = threadIdx.x; i < n; i += blockDim.x) progress[i] = 0;
    if (failed && threadIdx.x == 0) *failed = 0;      // null: keep what an earlier launch of this plan reported
}

__global__ __launch_bounds__(kCopyThreads) void slide_down(char *dst, const char *src, uint64_t len,
                                                           uint32_t *progress, uint32_t *failed,
                                                           uint32_t spin_limit)
{
    const uint64_t shift = (uint64_t)(src - dst);
    const uint64_t chunks = (len + kSlideChunk - 1) / kSlideChunk;
    const uint64_t q = shift / kSlideChunk;
    const bool straddles = shift % kSlideChunk != 0;
    const uint32_t G = gridDim.x, w = blockIdx.x;
    __shared__ uint32_t give_up;
    uint32_t round = 0;
    for (uint64_t chunk = w; chunk < chunks; chunk += G, ++round) {
        const uint64_t off = chunk * kSlideChunk;
        const uint64_t left = len - off;
        const uint32_t nvec = (uint32_t)((left < kSlideChunk ? left : kSlideChunk) / 16);
        const u32x4 *s = (const u32x4 *)(src + off);
        u32x4 *d = (u32x4 *)(dst + off);
        u32x4 v[kSlideVec];
#pragma unroll
        for (int j = 0; j < kSlideVec; ++j) {
            const uint32_t i = threadIdx.x + j * kCopyThreads;
            if (i < nvec) v[j] = __builtin_nontemporal_load(s + i);
        }
        // all loads of this workgroup have returned before the counter moves
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (threadIdx.x == 0) {
            __hip_atomic_store(progress + w, round + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            // chunks whose source this chunk's destination covers (other than itself)
            uint32_t bad = 0;
            const uint64_t need[2] = {chunk - q - 1, chunk - q};
            const bool want[2] = {straddles && chunk >= q + 1, q > 0 && chunk >= q};
            for (int k = 0; k < 2 && !bad; ++k) {
                if (!want[k]) continue;
                const uint32_t owner = (uint32_t)(need[k] % G), target = (uint32_t)(need[k] / G) + 1;
                uint32_t spins = 0;
                while (__hip_atomic_load(progress + owner, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
                    if (++spins > spin_limit) { bad = 1; break; }
                    __builtin_amdgcn_s_sleep(4);
                }
            }
            if (bad) __hip_atomic_store(failed, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            give_up = bad;
        }
        __syncthreads();
        if (!give_up) {
#pragma unroll
            for (int j = 0; j < kSlideVec; ++j) {
                const uint32_t i = threadIdx.x + j * kCopyThreads;
                if (i < nvec) __builtin_nontemporal_store(v[j], d + i);
            }
        }
        __syncthreads();            // give_up is rewritten in the next round
    }
}

static hipError_t launch_slide_down(char *dst, const char *src, uint64_t len, SlideState *st, bool clear_failed,
                                    hipStream_t stream)
{
    if (!st || !st->progress) return hipErrorInvalidValue;
    const uint64_t chunks = (len + kSlideChunk - 1) / kSlideChunk;
    if (st->max_grid == 0) {
        int per_cu = 0, dev = 0, cus = 0;
        hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, slide_down, kCopyThreads, 0);
        if (e == hipSuccess) e = hipGetDevice(&dev);
        if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return e;
        if (per_cu < 1 || cus < 1) return hipErrorInvalidValue;
        // two workgroups per compute unit keep 256 KB per unit in flight; more changes nothing
        st->max_grid = (uint32_t)std::min<int64_t>((int64_t)std::min(per_cu, 2) * cus, kSlideMaxGrid);
    }
    uint32_t grid = (uint32_t)std::min<uint64_t>(chunks, st->max_grid);
    hipLaunchKernelGGL(slide_reset, dim3(1), dim3(256), 0, stream, st->progress, grid,
                       clear_failed ? st->failed : (uint32_t *)nullptr);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(slide_down, dim3(grid), dim3(kCopyThreads), 0, stream, dst, (const char *)src, len,
                       st->progress, st->failed, st->spin_limit);
    return hipGetLastError();
}

hipError_t slide_state_create(SlideState *st)
{
    st->max_grid = 0;
    hipError_t e = hipMalloc((void **)&st->progress, (kSlideMaxGrid + 64) * sizeof(uint32_t));
    if (e != hipSuccess) { st->progress = nullptr; return e; }
    st->failed = st->progress + kSlideMaxGrid;
    return hipMemset(st->progress, 0, (kSlideMaxGrid + 64) * sizeof(uint32_t));
}

void slide_state_destroy(SlideState *st)
{
    if (st->progress) (void)hipFree(st->progress);
    st->progress = st->failed = nullptr;
}

// 1 if a slide launched since the last call gave up a wait (the caller has synchronized).
hipError_t slide_state_failed(SlideState *st, hipStream_t stream, uint32_t *out)
{
    *out = 0;
    if (!st->progress) return hipSuccess;
    hipError_t e = hipMemcpyAsync(out, st->failed, 4, hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    // reported once: a later plan without an in-place move must not see it again
    if (e == hipSuccess && *out) e = hipMemsetAsync(st->failed, 0, 4, stream);
    return e;
}

// Sliding compaction.  Moves are listed in ascending address order and every
// destination lies below its source.  A move whose shift (src - dst) is at
// least its length is an independent segment; consecutive ones share a launch as
// long as none of them writes what an earlier one of the same launch still reads.
// A move that overlaps its own destination runs as one in-place slide_down launch.
// Launches run in stream order.
hipError_t launch_slide(char *base, const uint64_t *src, const uint64_t *dst, const uint64_t *len,
                        uint32_t n, SlideState *st, hipStream_t stream, uint64_t *launches)
{
    std::vector<CopySeg> phase;
    uint64_t phase_first_src = 0;
    bool first_slide = true;        // the plan's first in-place move clears the "gave up" flag, later ones keep it
    auto flush = [&]() -> hipError_t {
        if (phase.empty()) return hipSuccess;
        hipError_t e = launch_copy(phase.data(), (uint32_t)phase.size(), stream);
        if (launches) *launches += (phase.size() + kMaxSeg - 1) / kMaxSeg;
        phase.clear();
        return e;
    };
    for (uint32_t i = 0; i < n; ++i) {
        if (len[i] == 0) continue;
        const uint64_t shift = src[i] - dst[i];
        if (shift >= len[i]) {
            // joins the current launch only if it writes nothing that launch still reads
            if (!phase.empty() && dst[i] + len[i] > phase_first_src)
                if (hipError_t e = flush()) return e;
            if (phase.empty()) phase_first_src = src[i];
            phase.push_back({base + src[i], base + dst[i], len[i]});
            continue;
        }
        if (hipError_t e = flush()) return e;
        if (hipError_t e = launch_slide_down(base + dst[i], base + src[i], len[i], st, first_slide, stream))
            return e;
        first_slide = false;
        if (launches) *launches += 1;
    }
    return flush();
}

// Exclusive prefix sum of up to 4096 integers with one workgroup: each
// wavefront scans 64 values at a time and carries its running total.
__global__ __launch_bounds__(64) void scan_u64(const uint64_t *in, uint32_t n, uint64_t *out)
{
    uint64_t carry = 0;
    for (uint32_t at = 0; at < n; at += 64) {
        const uint32_t i = at + threadIdx.x;
        const uint64_t v = i < n ? in[i] : 0;
        uint64_t total;
        const uint64_t e = wave_excl_scan_u64(v, &total);
        if (i < n) out[i] = carry + e;
        carry += total;
    }
    if (threadIdx.x == 0) out[n] = carry;
}

hipError_t launch_scan_u64(const uint64_t *dev_in, uint32_t n, uint64_t *dev_out, hipStream_t s)
{
    hipLaunchKernelGGL(scan_u64, dim3(1), dim3(64), 0, s, dev_in, n, dev_out);
    return hipGetLastError();
}

// Test pattern: word i of a range holds mix(seed + i * odd constant) with the
// splitmix64 finalizer, so any part of a huge range can be verified on its own.
__device__ __host__ inline uint64_t pattern_word(uint64_t seed, uint64_t i)
{
    uint64_t z = seed + i * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__global__ __launch_bounds__(256) void fill_pattern(uint64_t *p, uint64_t nwords, uint64_t seed)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nwords; i += stride)
        p[i] = pattern_word(seed, i);
}

__global__ __launch_bounds__(256) void check_pattern(const uint64_t *p, uint64_t nwords,
                                                     uint64_t seed, unsigned long long *bad)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    unsigned long long mine = 0;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nwords; i += stride)
        mine += p[i] != pattern_word(seed, i);
    if (mine) atomicAdd(bad, mine);
}

// Calibration: nothing but loads.  Every workgroup reads 256 KiB in one piece, a wavefront
// instruction 1 KiB, eight instructions in flight per wavefront, non-temporal: what the
// memory system delivers to a kernel that only streams (sink is written only if the data
// xor to a value they never have).
__global__ __launch_bounds__(256) void read_only(const char *base, uint64_t nbytes, u32x4 *sink)
{
    constexpr uint64_t kPiece = 256 * 1024;
    const uint64_t off = (uint64_t)blockIdx.x * kPiece;
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint64_t left = nbytes - off;
    const uint32_t n = (uint32_t)((left < kPiece ? left : kPiece) / 4096);      // whole 4 KiB steps of the workgroup
    const char *p = base + off + wave * 1024 + lane * 16;
    u32x4 acc = {0u, 0u, 0u, 0u};
    uint32_t i = 0;
    for (; i + 8 <= n; i += 8) {
        u32x4 v[8];
#pragma unroll
        for (int d = 0; d < 8; ++d) v[d] = __builtin_nontemporal_load((const u32x4 *)(p + (uint64_t)(i + d) * 4096));
#pragma unroll
        for (int d = 0; d < 8; ++d) acc ^= v[d];
    }
    for (; i < n; ++i) acc ^= __builtin_nontemporal_load((const u32x4 *)(p + (uint64_t)i * 4096));
    if (acc[0] == 0x9e3779b9u && acc[1] == 0x7f4a7c15u && acc[2] == 0xf39cc060u && acc[3] == 0x5cedc834u) *sink = acc;
}

// nbytes: a multiple of 4096; sink: 16 device bytes
hipError_t launch_read_only(const void *dev, uint64_t nbytes, void *sink, hipStream_t s)
{
    const uint64_t pieces = (nbytes + 256 * 1024 - 1) / (256 * 1024);
    if (!pieces) return hipSuccess;
    if (pieces > 0x7fffffffull) return hipErrorInvalidValue;
    hipLaunchKernelGGL(read_only, dim3((uint32_t)pieces), dim3(256), 0, s, (const char *)dev, nbytes, (u32x4 *)sink);
    return hipGetLastError();
}

hipError_t launch_fill_pattern(void *dev, uint64_t nbytes, uint64_t seed, hipStream_t s)
{
    const uint64_t nwords = nbytes / 8;
    if (!nwords) return hipSuccess;
    const uint32_t grid = (uint32_t)std::min<uint64_t>((nwords + 255) / 256, 256 * 32);
    hipLaunchKernelGGL(fill_pattern, dim3(grid), dim3(256), 0, s, (uint64_t *)dev, nwords, seed);
    return hipGetLastError();
}

hipError_t launch_check_pattern(const void *dev, uint64_t nbytes, uint64_t seed,
                                unsigned long long *dev_bad, hipStream_t s)
{
    const uint64_t nwords = nbytes / 8;
    if (!nwords) return hipSuccess;
    const uint32_t grid = (uint32_t)std::min<uint64_t>((nwords + 255) / 256, 256 * 32);
    hipLaunchKernelGGL(check_pattern, dim3(grid), dim3(256), 0, s, (const uint64_t *)dev, nwords,
                       seed, dev_bad);
    return hipGetLastError();
}

}  // namespace salus
