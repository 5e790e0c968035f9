// Wavefront-level (64-lane) primitives shared by the kernels.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace salus {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Exclusive prefix sum across the 64 lanes of a wavefront (Hillis-Steele over
// cross-lane shuffles).  *total receives the sum over all lanes.
__device__ inline uint64_t wave_excl_scan_u64(uint64_t v, uint64_t *total)
{
    const int lane = threadIdx.x & 63;
    uint64_t incl = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint64_t up = __shfl_up((unsigned long long)incl, d, 64);
        if (lane >= d) incl += up;
    }
    if (total) *total = __shfl((unsigned long long)incl, 63, 64);
    return incl - v;
}

__device__ inline uint32_t wave_excl_scan_u32(uint32_t v, uint32_t *total)
{
    const int lane = threadIdx.x & 63;
    uint32_t incl = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint32_t up = __shfl_up(incl, d, 64);
        if (lane >= d) incl += up;
    }
    if (total) *total = __shfl(incl, 63, 64);
    return incl - v;
}

// Index of the lane whose half-open range [excl, excl + count) contains x, given
// each lane's exclusive prefix and the number of valid lanes.  Lanes with an
// empty range never win.  x must be below the total.
__device__ inline int wave_find_range(uint64_t excl, uint64_t x, bool valid)
{
    unsigned long long m = __ballot(valid && excl <= x);
    return 63 - __clzll((long long)m);
}

}  // namespace salus
