// One output tile of a dense layer, computed by a workgroup of four wavefronts:
// the arithmetic shared by the per-depth grouped kernels and the depth-fused ones.
#pragma once
#include "group.hpp"

namespace salus {

// Combine the four wavefronts' partial tiles.  Accumulator register r (0..3)
// of every 16x16 block holds row 4*(lane/16)+r, so wavefront w ends up owning
// rows with r == w: each wavefront sends the other three quarters through LDS
// and adds what it receives in a fixed order.
template <int NACC>
__device__ inline void reduce_scatter(f32x4 (&acc)[NACC], float (&own)[NACC], float *lds)
{
    constexpr int G = NACC < 16 ? NACC : 16;    // accumulators per pass (bounds the LDS footprint)
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // lds[dst wave][source slot][accumulator in pass][lane]
#pragma unroll
    for (int base = 0; base < NACC; base += G) {
        if (base) __syncthreads();              // the previous pass has been read
#pragma unroll
        for (int d = 0; d < kWaves; ++d) {
            if (d == wave) continue;
            const int slot = (wave - d - 1) & 3;
            float *to = lds + ((d * 3 + slot) * G) * 64 + lane;
#pragma unroll
            for (int i = 0; i < G; ++i) to[i * 64] = acc[base + i][d];
        }
        __syncthreads();
        const float *from = lds + (wave * 3 * G) * 64 + lane;
#pragma unroll
        for (int i = 0; i < G; ++i) {
            const f32x4 mine = acc[base + i];
            float v = wave == 0 ? mine[0] : wave == 1 ? mine[1] : wave == 2 ? mine[2] : mine[3];
            v += from[(0 * G + i) * 64];
            v += from[(1 * G + i) * 64];
            v += from[(2 * G + i) * 64];
            own[base + i] = v;
        }
    }
}

template <int NACC>
constexpr int reduce_lds_floats() { return kWaves * 3 * (NACC < 16 ? NACC : 16) * 64; }

// ---------------------------------------------------------------------------
// bf16 weights and activations, float accumulation, v_mfma_f32_16x16x32_bf16.
// Tile: TM = 16*MT rows x 128 columns.  Lane (c = lane%16, g = lane/16) of a
// wavefront loads, per k-step of 32 rows, the 8x8 block W[k0+8g .. +7][n0+8c ..
// +7] (eight 16-byte loads, 256 contiguous bytes per row across the 16 lanes)
// and transposes it in registers; column i of the block is the B operand of
// MFMA i, whose 16 output columns are n0 + 8c + i.  The A operand is
// X[m0 + c][k0+8g .. +7].  Both operands use the same 8 k-values per lane
// group, which is all the MFMA contraction needs.
// TW (backward pass, dX = dY . W^T): W is stored N x K, so the eight k-values of
// output column n0+8c+i are contiguous in row n0+8c+i and are loaded as they are.
// ---------------------------------------------------------------------------
// NT: every weight is read by one workgroup only (each job has a single row tile),
// so the loads carry the non-temporal hint and do not displace activations in
// L2.  With several row tiles per column tile the neighbours read the same
// weights at about the same time and a plain load lets the second one hit in L2.
template <int MT, bool TW, bool NT>
__device__ inline void dense_bf16_tile(const Problem &p, const Tile tile, float *lds)
{
    constexpr int NACC = MT * 8;
    const uint32_t M = p.M, K = p.K, N = p.N;
    const int lane = threadIdx.x & 63, c = lane & 15, g = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t ncol = tile.n0 + 8 * c;
    const bool col_ok = ncol < N;
    const uint16_t *W = (const uint16_t *)p.W;
    const uint16_t *X = (const uint16_t *)p.X;

    f32x4 acc[NACC];
#pragma unroll
    for (int i = 0; i < NACC; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int nsteps = (int)((K + 31) / 32);
    const u32x4 zero = {0u, 0u, 0u, 0u};

    // Loads are never predicated: a lane whose block lies outside the matrix
    // reads a clamped, valid address instead and its values are dropped later
    // (rows >= M and columns >= N are never stored; k-groups >= K get a zero A
    // operand).  With no branch around any load the compiler can count exactly
    // how many loads may stay in flight at each use, which is what keeps the
    // next step's loads outstanding while this step is multiplied.
    const uint32_t ncol_c = col_ok ? ncol : 0u;
    // Row-major W: row pitch N.  Strip layout: the 128 columns of this tile are one
    // contiguous K x 128 block (pitch 128), so a wavefront's k-step is 8 KB in one piece.
    const bool blocked_in = !TW && (p.flags & kInBlocked);     // implies M <= 32, so tile.m0 == 0
    const uint32_t xtiles = (M + 15) / 16;
    const bool strip = !TW && (p.flags & kStripW);
    const uint32_t wpitch = strip ? 128u : N;
    const uint16_t *Wc = strip ? W + (size_t)tile.n0 * K + 8 * c : W + ncol_c;
    auto load = [&](int s, u32x4 (&w)[8], u32x4 (&x)[MT], bool &k_ok) {
        const uint32_t kb = 32u * (uint32_t)s + 8u * (uint32_t)g;
        k_ok = kb < K;
        const uint32_t kc = k_ok ? kb : 0u;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const uint16_t *at = TW ? W + (size_t)(ncol_c + r) * K + kc : Wc + (size_t)(kc + r) * wpitch;
            w[r] = NT ? __builtin_nontemporal_load((const u32x4 *)at) : *(const u32x4 *)at;
        }
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            if (blocked_in) {
                // one contiguous kilobyte per wavefront; a row tile the job does not
                // have (its rows are never stored) reads the job's last one instead
                const uint32_t tt = (uint32_t)t < xtiles ? (uint32_t)t : xtiles - 1;
                x[t] = *(const u32x4 *)(X + (((size_t)(kc >> 5) * xtiles + tt) * 64 + lane) * 8);
            } else {
                const uint32_t row = tile.m0 + 16 * t + c;
                x[t] = *(const u32x4 *)(X + (size_t)(row < M ? row : M - 1) * K + kc);
            }
        }
    };
    auto compute = [&](const u32x4 (&w)[8], const u32x4 (&xr)[MT], bool k_ok) {
        u32x4 x[MT];
#pragma unroll
        for (int t = 0; t < MT; ++t) x[t] = k_ok ? xr[t] : zero;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            // column i of the 8x8 block: dword j = (row 2j, row 2j+1)
            u32x4 b;
            if (TW) {
                b = w[i];
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    b[j] = __builtin_amdgcn_perm(w[2 * j + 1][i >> 1], w[2 * j][i >> 1],
                                                 (i & 1) ? 0x07060302u : 0x05040100u);
            }
#pragma unroll
            for (int t = 0; t < MT; ++t)
                acc[t * 8 + i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                    __builtin_bit_cast(bf16x8, x[t]), __builtin_bit_cast(bf16x8, b), acc[t * 8 + i],
                    0, 0, 0);
        }
    };

    // The four wavefronts take k-steps wave, wave+4, ...: this wavefront owns
    // `mine` steps.  Two steps are in flight at any time; the last (up to three)
    // steps are peeled so that the main loop never loads past the end.
    u32x4 w0[8], w1[8], x0[MT], x1[MT];
    bool ok0, ok1;
    const int mine = nsteps > wave ? (nsteps - wave + kWaves - 1) / kWaves : 0;
    auto step = [&](int i) { return wave + kWaves * i; };
    load(step(0), w0, x0, ok0);
    load(step(1), w1, x1, ok1);
    int i = 0;
    for (; i + 3 < mine; i += 2) {
        // keep the instruction scheduler from sinking the loads below the next
        // multiply phase: each phase must stay where it is written
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

    const uint32_t act = p.flags & 0xffu;
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        const uint32_t row = tile.m0 + 16 * t + 4 * g + wave;
        if (row >= M || !col_ok) continue;
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = activate(own[t * 8 + i], act);
        if (p.flags & kMaskPositive) {
            // ReLU derivative taken from the stored bf16 activation (sign bit clear, not zero)
            const u32x4 h = *(const u32x4 *)((const uint16_t *)p.aux + (size_t)row * N + ncol);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t bits = (h[i >> 1] >> ((i & 1) * 16)) & 0xffffu;
                if ((bits & 0x8000u) || !(bits & 0x7fffu)) v[i] = 0.0f;
            }
        }
        if (p.flags & kOutBf16) {
            u32x4 o;
#pragma unroll
            for (int j = 0; j < 4; ++j) o[j] = bf16_pack(v[2 * j], v[2 * j + 1]);
            if (p.flags & kOutBlocked) {
                // these 8 columns are k-group (ncol / 8) % 4 of k-step ncol / 32 of the next layer
                const size_t unit = (((size_t)(ncol >> 5) * xtiles + (row >> 4)) * 4 + ((ncol >> 3) & 3)) * 16 +
                                    (row & 15);
                *(u32x4 *)((uint16_t *)p.Y + unit * 8) = o;
            } else {
                *(u32x4 *)((uint16_t *)p.Y + (size_t)row * N + ncol) = o;
            }
        } else {
            float *y = (float *)p.Y + (size_t)row * N + ncol;
            *(f32x4 *)y = f32x4{v[0], v[1], v[2], v[3]};
            *(f32x4 *)(y + 4) = f32x4{v[4], v[5], v[6], v[7]};
        }
    }
}

// ---------------------------------------------------------------------------
// float weights and activations, v_mfma_f32_16x16x4_f32 (true fp32 products).
// Tile: 16*MT rows x 64 columns; a k-step covers 16 rows of W.  Lane (c, g)
// loads W[k0+4g+q][n0+4c .. +3] for q = 0..3 and X[m0+c][k0+4g .. +3]; MFMA
// (q, i) multiplies component q of X with component i of W row q, so lane
// group g contributes k = k0+4g+q in step q and output column n0+4c+i.
// ---------------------------------------------------------------------------
template <int MT>
__device__ inline void dense_f32_tile(const Problem &p, const Tile tile, float *lds)
{
    constexpr int NACC = MT * 4;
    const uint32_t M = p.M, K = p.K, N = p.N;
    const int lane = threadIdx.x & 63, c = lane & 15, g = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t ncol = tile.n0 + 4 * c;
    const bool col_ok = ncol < N;
    const float *W = (const float *)p.W;
    const float *X = (const float *)p.X;

    f32x4 acc[NACC];
#pragma unroll
    for (int i = 0; i < NACC; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int nsteps = (int)((K + 15) / 16);
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};

    // unpredicated loads from clamped addresses, as in the bf16 kernel
    const uint32_t ncol_c = col_ok ? ncol : 0u;
    auto load = [&](int s, f32x4 (&w)[4], f32x4 (&x)[MT], bool &k_ok) {
        const uint32_t kb = 16u * (uint32_t)s + 4u * (uint32_t)g;
        k_ok = kb < K;
        const uint32_t kc = k_ok ? kb : 0u;
#pragma unroll
        for (int q = 0; q < 4; ++q) w[q] = *(const f32x4 *)(W + (size_t)(kc + q) * N + ncol_c);
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            const uint32_t row = tile.m0 + 16 * t + c;
            x[t] = *(const f32x4 *)(X + (size_t)(row < M ? row : M - 1) * K + kc);
        }
    };
    auto compute = [&](const f32x4 (&w)[4], const f32x4 (&xr)[MT], bool k_ok) {
        f32x4 x[MT];
#pragma unroll
        for (int t = 0; t < MT; ++t) x[t] = k_ok ? xr[t] : zero;
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int t = 0; t < MT; ++t)
                    acc[t * 4 + i] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[t][q], w[q][i],
                                                                          acc[t * 4 + i], 0, 0, 0);
    };

    f32x4 w0[4], w1[4], x0[MT], x1[MT];
    bool ok0, ok1;
    const int mine = nsteps > wave ? (nsteps - wave + kWaves - 1) / kWaves : 0;
    auto step = [&](int i) { return wave + kWaves * i; };
    load(step(0), w0, x0, ok0);
    load(step(1), w1, x1, ok1);
    int i = 0;
    for (; i + 3 < mine; i += 2) {
        // keep the instruction scheduler from sinking the loads below the next
        // multiply phase: each phase must stay where it is written
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

    const uint32_t act = p.flags & 0xffu;
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        const uint32_t row = tile.m0 + 16 * t + 4 * g + wave;
        if (row >= M || !col_ok) continue;
        f32x4 o;
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = activate_f32(own[t * 4 + i], act);
        *(f32x4 *)((float *)p.Y + (size_t)row * N + ncol) = o;
    }
}

}  // namespace salus
