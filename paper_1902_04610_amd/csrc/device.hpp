// Launchers of the gfx950 kernels (implemented in the .hip files).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace salus {

// ---- copy / compaction ----------------------------------------------------
struct CopySeg {
    const void *src;
    void *dst;
    uint64_t len;        // bytes, multiple of 16; src and dst 16-byte aligned
};
constexpr uint32_t kMaxSeg = 64;            // segments per launch (one per wavefront lane)
constexpr uint32_t kCopyChunk = 64 * 1024;  // bytes one workgroup moves per grid-stride step

// Copies n mutually independent segments (no destination may overlap another
// segment's source); more than kMaxSeg segments are split over launches.
hipError_t launch_copy(const CopySeg *segs, uint32_t n, hipStream_t stream);

// memmove toward lower addresses inside one allocation: dst < src, any overlap.
// bounce/bounce_len: a free device range usable as staging (may be empty).
hipError_t launch_slide(char *base, const uint64_t *src, const uint64_t *dst, const uint64_t *len,
                        uint32_t n, uint64_t bounce_off, uint64_t bounce_len, hipStream_t stream,
                        uint64_t *launches);

hipError_t launch_scan_u64(const uint64_t *dev_in, uint32_t n, uint64_t *dev_out, hipStream_t s);
hipError_t launch_fill_pattern(void *dev, uint64_t nbytes, uint64_t seed, hipStream_t s);
hipError_t launch_check_pattern(const void *dev, uint64_t nbytes, uint64_t seed,
                                unsigned long long *dev_bad, hipStream_t s);

// ---- grouped GEMM -----------------------------------------------------------
struct Problem {
    const void *W;       // K x N row-major
    const void *X;       // M x K row-major
    void *Y;             // M x N row-major
    uint32_t M, K, N;
    uint32_t flags;      // bits 0-7 activation, bit 8: store Y as bf16
};
constexpr uint32_t kMaxProblems = 64;       // problems per launch (one per wavefront lane)
constexpr uint32_t kOutBf16 = 1u << 8;

// One launch (or several when n > kMaxProblems): Y_g = act(X_g . W_g) for all g.
hipError_t launch_grouped_bf16(const Problem *p, uint32_t n, hipStream_t stream, uint64_t *launches);
hipError_t launch_grouped_f32(const Problem *p, uint32_t n, hipStream_t stream, uint64_t *launches);

}  // namespace salus
