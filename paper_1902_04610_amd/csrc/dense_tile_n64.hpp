// A 16*MT x 64 output tile of a bf16 dense layer, computed by four wavefronts:
// the narrow-tile variant of dense_bf16_tile for jobs of 33 .. 64 rows.
//
// Why it exists.  The weight stream of one compute unit is limited (about 30 GB/s
// on MI355X in this access pattern, measured: 32, 64 or 128 workgroups of the
// wide kernel each need the same 20 us for a 2048-deep layer, and a launch only
// approaches the HBM rate when all 256 compute units stream).  Two consequences
// for jobs of up to 64 rows: (1) the weights must pass through a compute unit's
// vector memory path once, so one workgroup holds all 64 rows (MT = 4) instead
// of two 32-row workgroups that both load W, the second from L2; (2) a launch
// needs as many workgroups as compute units even when it holds few jobs, so the
// column tile is 64 wide, which doubles the workgroup count.
//
// Mapping.  v_mfma_f32_16x16x32_bf16 wants, from lane (n = lane % 16, g = lane / 16),
// eight k-values of output column n.  A lane still loads an 8 x 8 block of W
// (eight 16-byte loads) and transposes it in registers, which yields eight
// columns, but a 64-column tile only has 8 column blocks for 16 lanes.  So a
// k-step covers 64 rows of W and the two halves of a 16-lane row take different
// k: lane (cb = n % 8, h = n / 8, g) loads rows k0 + 16 g + 8 h .. + 7 of columns
// n0 + 8 cb .. + 7.  The step is multiplied as two sub-steps (h' = 0, 1; k-group g
// of sub-step h' is k0 + 16 g + 8 h' .. + 7).  In sub-step h' the lanes with
// h == h' hold the operand for their own column block; the other eight lanes of
// the row need the same blocks, and take the odd (h' = 0) or even (h' = 1)
// columns from their partner lane n ^ 8 with one DPP row rotation per dword.
// MFMA i' (0..3) thus computes columns {8 cb + 2 i' (lanes n < 8), 8 cb + 2 i' + 1
// (lanes n >= 8)}: no multiply is wasted, and both activation sub-step loads of a
// lane are adjacent 16-byte pieces of one row.
// TW (dX = dY . W^T): W is stored N x K; the eight k-values of output column
// n0 + 8 cb + j are contiguous in W's row n0 + 8 cb + j and are loaded as they are;
// the partner exchange is the same.
#pragma once
#include "dense_tile.hpp"

namespace salus {

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

// lanes 8..15 of every 16-lane row receive `odd` from lane - 8, lanes 0..7 keep `even`
__device__ inline uint32_t take_partner_hi(uint32_t even, uint32_t odd)
{
    return (uint32_t)__builtin_amdgcn_update_dpp((int)even, (int)odd, 0x128 /* row_ror:8 */, 0xf, 0xc, false);
}
// lanes 0..7 receive `even` from lane + 8, lanes 8..15 keep `odd`
__device__ inline uint32_t take_partner_lo(uint32_t odd, uint32_t even)
{
    return (uint32_t)__builtin_amdgcn_update_dpp((int)odd, (int)even, 0x128 /* row_ror:8 */, 0xf, 0x3, false);
}
__device__ inline float swap_partner(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x128, 0xf, 0xf, false));
}

template <int MT, bool TW, bool NT>
__device__ inline void dense_bf16_tile_n64(const Problem &p, const Tile tile, float *lds)
{
    constexpr int NACC = MT * 4;
    const uint32_t M = p.M, K = p.K, N = p.N;
    const int lane = threadIdx.x & 63, c = lane & 15, g = lane >> 4, cb = c & 7, h = c >> 3;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t nblk = tile.n0 + 8 * cb;         // first column of this lane's block
    const bool blk_ok = nblk < N;
    const uint16_t *W = (const uint16_t *)p.W;
    const uint16_t *X = (const uint16_t *)p.X;

    f32x4 acc[NACC];
#pragma unroll
    for (int i = 0; i < NACC; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int nsteps = (int)((K + 63) / 64);
    const u32x4 zero = {0u, 0u, 0u, 0u};
    // unpredicated loads from clamped addresses (see dense_bf16_tile)
    const uint32_t nblk_c = blk_ok ? nblk : 0u;
    const bool strip = !TW && (p.flags & kStripW);
    const uint32_t wpitch = strip ? 128u : N;
    const uint16_t *Wc = strip ? W + (size_t)(tile.n0 >> 7) * K * 128 + (tile.n0 & 127u) + 8 * cb : W + nblk_c;

    auto load = [&](int s, u32x4 (&w)[8], u32x4 (&x)[MT][2], uint32_t &k_ok) {
        const uint32_t kg = 64u * (uint32_t)s + 16u * (uint32_t)g;     // this k-group: kg + 8 h' .. + 7
        const uint32_t kb = kg + 8u * (uint32_t)h;                     // this lane's rows of W
        const uint32_t kc = kb < K ? kb : 0u;
        k_ok = (kg < K ? 1u : 0u) | (kg + 8u < K ? 2u : 0u);
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const uint16_t *at = TW ? W + (size_t)(nblk_c + r) * K + kc : Wc + (size_t)(kc + r) * wpitch;
            w[r] = NT ? __builtin_nontemporal_load((const u32x4 *)at) : *(const u32x4 *)at;
        }
        const uint32_t kx = kg < K ? kg : 0u;
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            const uint32_t row = tile.m0 + 16 * t + c;
            const uint16_t *xr = X + (size_t)(row < M ? row : M - 1) * K + kx;
            x[t][0] = *(const u32x4 *)xr;
            x[t][1] = *(const u32x4 *)(xr + (kg + 8u < K ? 8 : 0));
        }
    };
    auto compute = [&](const u32x4 (&w)[8], const u32x4 (&xr)[MT][2], uint32_t k_ok) {
        u32x4 x[MT][2];
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            x[t][0] = (k_ok & 1u) ? xr[t][0] : zero;
            x[t][1] = (k_ok & 2u) ? xr[t][1] : zero;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            // columns 2i and 2i+1 of the lane's 8x8 block: dword q = (row 2q, row 2q+1)
            u32x4 even, odd;
            if (TW) {
                even = w[2 * i];
                odd = w[2 * i + 1];
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    even[q] = __builtin_amdgcn_perm(w[2 * q + 1][i], w[2 * q][i], 0x05040100u);
                    odd[q] = __builtin_amdgcn_perm(w[2 * q + 1][i], w[2 * q][i], 0x07060302u);
                }
            }
            u32x4 b0, b1;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                b0[q] = take_partner_hi(even[q], odd[q]);      // sub-step 0: data of the h = 0 lanes
                b1[q] = take_partner_lo(odd[q], even[q]);      // sub-step 1: data of the h = 1 lanes
            }
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                acc[t * 4 + i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                    __builtin_bit_cast(bf16x8, x[t][0]), __builtin_bit_cast(bf16x8, b0), acc[t * 4 + i], 0, 0, 0);
                acc[t * 4 + i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                    __builtin_bit_cast(bf16x8, x[t][1]), __builtin_bit_cast(bf16x8, b1), acc[t * 4 + i], 0, 0, 0);
            }
        }
    };

    // k-steps wave, wave + 4, ...; two in flight; the tail is peeled (see dense_bf16_tile)
    u32x4 w0[8], w1[8], x0[MT][2], x1[MT][2];
    uint32_t ok0, ok1;
    const int mine = nsteps > wave ? (nsteps - wave + kWaves - 1) / kWaves : 0;
    auto step = [&](int i) { return wave + kWaves * i; };
    load(step(0), w0, x0, ok0);
    load(step(1), w1, x1, ok1);
    int i = 0;
    for (; i + 3 < mine; i += 2) {
        compute(w0, x0, ok0);
        __builtin_amdgcn_sched_barrier(0);
        load(step(i + 2), w0, x0, ok0);
        __builtin_amdgcn_sched_barrier(0);
        compute(w1, x1, ok1);
        __builtin_amdgcn_sched_barrier(0);
        load(step(i + 3), w1, x1, ok1);
        __builtin_amdgcn_sched_barrier(0);
    }
    const int left = mine - i;
    if (left >= 1) compute(w0, x0, ok0);
    if (left == 3) load(step(i + 2), w0, x0, ok0);
    if (left >= 2) compute(w1, x1, ok1);
    if (left == 3) compute(w0, x0, ok0);

    float own[NACC];
    reduce_scatter<NACC>(acc, own, lds);

    // own[t * 4 + i]: row m0 + 16 t + 4 g + wave, column 8 cb + 2 i + h.  The partner
    // lane holds the other parity of the same block; after the exchange a lane
    // has four consecutive columns: 8 cb + 4 h .. + 3.
    const uint32_t act = p.flags & 0xffu;
    const uint32_t ncol = nblk + 4u * (uint32_t)h;
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        // h = 0 keeps i = 0, 1 and needs the partner's i = 0, 1; h = 1 keeps i = 2, 3 and needs the partner's
        const float send0 = h ? own[t * 4 + 0] : own[t * 4 + 2];
        const float send1 = h ? own[t * 4 + 1] : own[t * 4 + 3];
        const float got0 = swap_partner(send0), got1 = swap_partner(send1);
        float v[4];
        if (h == 0) {
            v[0] = own[t * 4 + 0]; v[1] = got0; v[2] = own[t * 4 + 1]; v[3] = got1;
        } else {
            v[0] = got0; v[1] = own[t * 4 + 2]; v[2] = got1; v[3] = own[t * 4 + 3];
        }
        const uint32_t row = tile.m0 + 16 * t + 4 * g + wave;
        if (row >= M || !blk_ok) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = activate(v[j], act);
        if (p.flags & kMaskPositive) {
            // ReLU derivative taken from the stored bf16 activation (sign bit clear, not zero)
            const u32x2 hm = *(const u32x2 *)((const uint16_t *)p.aux + (size_t)row * N + ncol);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t bits = (hm[j >> 1] >> ((j & 1) * 16)) & 0xffffu;
                if ((bits & 0x8000u) || !(bits & 0x7fffu)) v[j] = 0.0f;
            }
        }
        if (p.flags & kOutBf16) {
            u32x2 o;
            o[0] = bf16_pack(v[0], v[1]);
            o[1] = bf16_pack(v[2], v[3]);
            *(u32x2 *)((uint16_t *)p.Y + (size_t)row * N + ncol) = o;
        } else {
            *(f32x4 *)((float *)p.Y + (size_t)row * N + ncol) = f32x4{v[0], v[1], v[2], v[3]};
        }
    }
}

}  // namespace salus
