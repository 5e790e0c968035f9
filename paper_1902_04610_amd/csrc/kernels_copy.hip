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

// Sliding compaction.  Moves are listed in ascending address order and every
// destination lies below its source.  A move whose shift (src - dst) is at
// least its length is one independent segment.  Otherwise it is cut into
// pieces no longer than the shift, so that each piece's destination ends where
// its source begins; pieces are then grouped into launches such that no
// destination written by a launch overlaps a source read by the same launch,
// and launches run in stream order.  When the shift is small the piece size
// would make the number of launches explode; such moves are staged through
// `bounce`, a free range above all live blocks (two copies per piece).
hipError_t launch_slide(char *base, const uint64_t *src, const uint64_t *dst, const uint64_t *len,
                        uint32_t n, uint64_t bounce_off, uint64_t bounce_len, hipStream_t stream,
                        uint64_t *launches)
{
    constexpr uint64_t kDirectMin = 32ull << 20;    // pieces at least this long run near full speed
    bounce_len &= ~(uint64_t)255;
    std::vector<CopySeg> phase;
    uint64_t phase_first_src = 0;
    auto flush = [&]() -> hipError_t {
        if (phase.empty()) return hipSuccess;
        hipError_t e = launch_copy(phase.data(), (uint32_t)phase.size(), stream);
        if (launches) *launches += (phase.size() + kMaxSeg - 1) / kMaxSeg;
        phase.clear();
        return e;
    };
    auto add = [&](uint64_t s, uint64_t d, uint64_t l) -> hipError_t {
        // joins the current launch only if it writes nothing that launch still reads
        if (!phase.empty() && d + l > phase_first_src)
            if (hipError_t e = flush()) return e;
        if (phase.empty()) phase_first_src = s;
        phase.push_back({base + s, base + d, l});
        return hipSuccess;
    };
    for (uint32_t i = 0; i < n; ++i) {
        const uint64_t shift = src[i] - dst[i];
        if (shift >= len[i]) {
            if (hipError_t e = add(src[i], dst[i], len[i])) return e;
            continue;
        }
        const bool direct = shift >= kDirectMin || shift >= bounce_len;
        if (direct) {
            for (uint64_t at = 0; at < len[i]; at += shift)
                if (hipError_t e = add(src[i] + at, dst[i] + at, std::min(shift, len[i] - at))) return e;
        } else {
            if (hipError_t e = flush()) return e;
            for (uint64_t at = 0; at < len[i]; at += bounce_len) {
                const uint64_t l = std::min(bounce_len, len[i] - at);
                CopySeg in{base + src[i] + at, base + bounce_off, l};
                CopySeg out{base + bounce_off, base + dst[i] + at, l};
                if (hipError_t e = launch_copy(&in, 1, stream)) return e;
                if (hipError_t e = launch_copy(&out, 1, stream)) return e;
                if (launches) *launches += 2;
            }
        }
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
