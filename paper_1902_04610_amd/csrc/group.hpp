// Pieces shared by the grouped dense kernels: the by-value argument block, the
// epilogue arithmetic and the workgroup -> (job, tile) lookup.
#pragma once
#include "device.hpp"
#include "wave.hpp"

namespace salus {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct GroupArgs {
    uint32_t n;
    uint32_t tiles;      // all tiles of the launch (kernels whose workgroups loop over tiles)
    Problem p[kMaxProblems];
};

constexpr int kGemmThreads = 256;
constexpr int kWaves = 4;

// bf16 kernels: GELU(z) = z / 2 + |z| (1/2 - Q(|z|)) with the upper tail Q(x) = erfc(x / sqrt 2) / 2
// taken from approximation 7.1.28 of Abramowitz & Stegun, erfc(y) = (1 + a1 y + ... + a6 y^6)^-16
// (absolute error below 3e-7, far inside half a bf16 step): the factors 1 / sqrt 2 of y and 2^(1/16) of
// the 1/2 are folded into the coefficients, so it is six multiply-adds, one reciprocal, four squarings
// and three more operations, no exponential and no branch (in float arithmetic over [-9, 9]: |error| of
// the result below 8e-7).  The error is *absolute* in Q, so for z < -3.5, where Q itself falls below
// 5e-4, the relative error of a single output grows - such outputs are below 1e-3 in magnitude and only
// decide a comparison when a whole matrix consists of them (then the error relative to the largest
// output is up to 2.3e-3, still inside the 2e-2 bound of the bf16 path).  Large |z| overflow the polynomial to
// infinity, whose reciprocal is the right Q = 0; a NaN stays a NaN.
__device__ inline float gelu_fast(float z)
{
    const float x = fabsf(z);
    float p = fmaf(5.62129980608006e-06f, x, 5.105520904180594e-05f);
    p = fmaf(p, x, 3.9686136005911976e-05f);
    p = fmaf(p, x, 0.003422739217057824f);
    p = fmaf(p, x, 0.02207699790596962f);
    p = fmaf(p, x, 0.052075162529945374f);
    p = fmaf(p, x, 1.0442737340927124f);
    float r = __frcp_rn(p);
    r *= r;
    r *= r;
    r *= r;
    r *= r;                                   // Q(|z|)
    return fmaf(x, 0.5f - r, 0.5f * z);
}

__device__ inline float activate(float z, uint32_t act)
{
    if (act == 1) return fmaxf(z, 0.0f);
    if (act == 2) return gelu_fast(z);
    return z;
}

// float kernels: the bound is relative (1e-5 of the largest output), so GELU is
// 0.5 z erfc(-z / sqrt 2) with the library's erfc, accurate to a few ulp in the
// negative tail as well.  These kernels are latency-bound; the cost does not show.
__device__ inline float activate_f32(float z, uint32_t act)
{
    if (act == 1) return fmaxf(z, 0.0f);
    if (act == 2) return 0.5f * z * erfcf(-0.70710678118654752440f * z);
    return z;
}

// float -> bf16 bits, round to nearest, ties to even (v_cvt_pk_bf16_f32).
__device__ inline uint32_t bf16_bits(float f)
{
    return __builtin_bit_cast(uint16_t, (__bf16)f);
}

// two floats -> two bf16 in one dword (a in the low half), one instruction
__device__ inline uint32_t bf16_pack(float a, float b)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{a, b}, bf16x2));
}

// Workgroups are dealt round-robin to the 8 XCDs (each with its own L2); map
// the hardware index to a logical one so that every XCD works on a contiguous
// range of tiles - the tiles of one job share its activations in one L2.
__device__ inline uint32_t xcd_remap(uint32_t b, uint32_t total)
{
    const uint32_t x = b & 7u, slot = b >> 3;
    const uint32_t q = total >> 3, r = total & 7u;
    return x * q + (x < r ? x : r) + slot;
}

struct Tile {
    int problem;
    uint32_t m0, n0;
};

// Which (job, row tile, column tile) this workgroup owns: lane i of every
// wavefront holds job i's tile count; an exclusive scan gives each job's first
// tile; a ballot finds the job whose range contains this workgroup's index.
template <int TM, int TN>
__device__ inline Tile find_tile(const GroupArgs &a)
{
    const int lane = threadIdx.x & 63;
    const bool valid = lane < (int)a.n;
    uint32_t row_tiles = 0, count = 0;
    if (valid) {
        row_tiles = (a.p[lane].M + TM - 1) / TM;
        count = row_tiles * ((a.p[lane].N + TN - 1) / TN);
    }
    const uint32_t first = wave_excl_scan_u32(count, nullptr);
    const uint32_t id = xcd_remap(blockIdx.x, gridDim.x);
    const int g = wave_find_range(first, id, valid);
    const uint32_t t = id - __shfl(first, g, 64);
    const uint32_t rt = __shfl(row_tiles, g, 64);
    Tile tile;
    tile.problem = __builtin_amdgcn_readfirstlane(g);
    tile.m0 = (t % rt) * TM;      // row tiles of one column tile are neighbours: they share W
    tile.n0 = (t / rt) * TN;
    return tile;
}

}  // namespace salus
