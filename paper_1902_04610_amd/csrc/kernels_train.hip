// Training-step kernels for gfx950: softmax cross-entropy with its gradient,
// and the fused weight-gradient + SGD update.  (The input-gradient product
// dX = dY . W^T reuses grouped_dense_bf16 with the transposed-weight load path.)
//
// A training iteration is a forward pass, a backward pass and a parameter
// update (Salus paper, Section 2.1); hyper-parameter tuning packs many such
// jobs of one architecture on a GPU (Section 5.2).  All jobs of a round share
// every launch here, as in the forward pass.
#include <algorithm>

#include "group.hpp"

namespace salus {

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

__device__ inline uint32_t bf16_rne(float f) { return bf16_bits(f); }

__device__ inline float wave_max(float v)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v = fmaxf(v, __shfl_xor(v, d, 64));
    return v;
}

__device__ inline float wave_sum(float v)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}

// ---------------------------------------------------------------------------
// Mean softmax cross-entropy over the M rows of each job and its gradient
// (softmax - onehot) / M, written as bf16 for the backward products.  A
// workgroup of 16 wavefronts takes 64 rows of one job (the job is found with the
// scan + ballot used everywhere else), one wavefront four rows.  Rows of up to
// 1024 classes are read once and kept in registers (all four rows' loads are in
// flight together); wider rows are re-read from memory for each of the three
// passes.  Row losses are added in row order by one thread, so the result does
// not depend on how the rows were scheduled: inside the workgroup when it holds
// the whole job, else by a second, tiny kernel over the scratch array.
// ---------------------------------------------------------------------------
struct LossArgs {
    uint32_t n;
    uint32_t pad;
    LossProblem p[kMaxProblems];
};

constexpr int kLossRows = 64, kLossWaves = 16, kLossPerWave = kLossRows / kLossWaves, kLossRegs = 16;

__global__ __launch_bounds__(64 * kLossWaves) void softmax_xent_rows(LossArgs a)
{
    __shared__ float row_loss[kLossRows];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool valid = lane < (int)a.n;
    const uint32_t blocks = valid ? (a.p[lane].M + kLossRows - 1) / kLossRows : 0;
    const uint32_t first = wave_excl_scan_u32(blocks, nullptr);
    const int job = __builtin_amdgcn_readfirstlane(wave_find_range(first, blockIdx.x, valid));
    const LossProblem &p = a.p[job];
    const uint32_t row0 = (blockIdx.x - __shfl(first, job, 64)) * kLossRows;
    const uint32_t M = p.M, N = p.N;
    const float inv_m = 1.0f / (float)M;
    // register path: lane owns classes 256 i + 4 lane .. + 3 of a row (16-byte loads, 8-byte stores)
    const bool in_regs = N <= 64u * kLossRegs && N % 4 == 0;

    f32x4 zr[kLossPerWave][kLossRegs / 4];
    int labels[kLossPerWave];
#pragma unroll
    for (int q = 0; q < kLossPerWave; ++q) {
        const uint32_t row = row0 + wave * kLossPerWave + q;
        const int l = p.labels[row < M ? row : M - 1];
        labels[q] = l < 0 ? 0 : (l >= (int)N ? (int)N - 1 : l);          // never read outside the row
    }
    if (in_regs) {
#pragma unroll
        for (int q = 0; q < kLossPerWave; ++q) {
            const uint32_t row = row0 + wave * kLossPerWave + q;
            const float *z = p.logits + (size_t)(row < M ? row : M - 1) * N;
#pragma unroll
            for (int i = 0; i < kLossRegs / 4; ++i) {
                const uint32_t n = 256u * i + 4u * lane;
                zr[q][i] = *(const f32x4 *)(z + (n < N ? n : N - 4));
            }
        }
    }
#pragma unroll
    for (int q = 0; q < kLossPerWave; ++q) {
        const uint32_t row = row0 + wave * kLossPerWave + q;
        if (row >= M) continue;                              // uniform per wavefront
        const float *z = p.logits + (size_t)row * N;
        uint16_t *g = (uint16_t *)p.grad + (size_t)row * N;
        const int label = labels[q];
        float zmax = -INFINITY, denom = 0.0f, zlabel = 0.0f;
        if (in_regs) {
#pragma unroll
            for (int i = 0; i < kLossRegs / 4; ++i)
                if (256u * i + 4u * lane < N)
                    zmax = fmaxf(fmaxf(zmax, fmaxf(zr[q][i][0], zr[q][i][1])), fmaxf(zr[q][i][2], zr[q][i][3]));
            zmax = wave_max(zmax);
            f32x4 e[kLossRegs / 4];
#pragma unroll
            for (int i = 0; i < kLossRegs / 4; ++i) {
                // v_exp_f32: error at the last-bit level, far below the bf16 rounding of the gradient
#pragma unroll
                for (int j = 0; j < 4; ++j) e[i][j] = __expf(zr[q][i][j] - zmax);
                if (256u * i + 4u * lane < N) denom += (e[i][0] + e[i][1]) + (e[i][2] + e[i][3]);
            }
            denom = wave_sum(denom);
            const float inv_d = 1.0f / denom;
#pragma unroll
            for (int i = 0; i < kLossRegs / 4; ++i) {
                const uint32_t n = 256u * i + 4u * lane;
                if (n >= N) continue;
                float h[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const bool hit = (int)(n + j) == label;
                    if (hit) zlabel = zr[q][i][j];
                    h[j] = (e[i][j] * inv_d - (hit ? 1.0f : 0.0f)) * inv_m;
                }
                *(u32x2 *)(g + n) = u32x2{bf16_pack(h[0], h[1]), bf16_pack(h[2], h[3])};
            }
            // the lane that holds the label's class hands its logit to lane 0
            zlabel = __shfl(zlabel, (label & 255) >> 2, 64);
        } else {
            for (uint32_t n = lane; n < N; n += 64) zmax = fmaxf(zmax, z[n]);
            zmax = wave_max(zmax);
            for (uint32_t n = lane; n < N; n += 64) denom += expf(z[n] - zmax);
            denom = wave_sum(denom);
            const float inv_d = 1.0f / denom;
            for (uint32_t n = lane; n < N; n += 64) {
                const float prob = expf(z[n] - zmax) * inv_d;
                g[n] = (uint16_t)bf16_rne((prob - ((int)n == label ? 1.0f : 0.0f)) * inv_m);
            }
        }
        if (!in_regs) zlabel = z[label];
        if (lane == 0) {
            const float loss = -(zlabel - zmax - logf(denom));
            row_loss[row - row0] = loss;
            if (M > (uint32_t)kLossRows) p.row_loss[row] = loss;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0 && M <= (uint32_t)kLossRows) {      // this workgroup holds the whole job
        float sum = 0.0f;
#pragma unroll
        for (uint32_t r = 0; r < (uint32_t)kLossRows; ++r) {
            const float v = row_loss[r < M ? r : 0];
            if (r < M) sum += v;
        }
        *p.loss = sum / (float)M;
    }
}

// Jobs of more than 64 rows: add the row losses of each in row order.
__global__ __launch_bounds__(64) void loss_mean(LossArgs a)
{
    const LossProblem &p = a.p[blockIdx.x];
    if (threadIdx.x != 0 || p.M <= (uint32_t)kLossRows) return;
    float sum = 0.0f;
    for (uint32_t r = 0; r < p.M; ++r) sum += p.row_loss[r];
    *p.loss = sum / (float)p.M;
}

hipError_t launch_softmax_xent(const LossProblem *p, uint32_t n, hipStream_t stream, uint64_t *launches)
{
    for (uint32_t at = 0; at < n; at += kMaxProblems) {
        LossArgs a{};
        a.n = std::min(kMaxProblems, n - at);
        uint64_t blocks = 0;
        bool big = false;
        for (uint32_t i = 0; i < a.n; ++i) {
            a.p[i] = p[at + i];
            blocks += (a.p[i].M + kLossRows - 1) / kLossRows;
            big = big || a.p[i].M > (uint32_t)kLossRows;
        }
        if (blocks == 0) continue;
        if (blocks > 0x7fffffffull) return hipErrorInvalidValue;
        hipLaunchKernelGGL(softmax_xent_rows, dim3((uint32_t)blocks), dim3(64 * kLossWaves), 0, stream, a);
        if (big) hipLaunchKernelGGL(loss_mean, dim3(a.n), dim3(64), 0, stream, a);
        if (launches) *launches += 1;
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// ---------------------------------------------------------------------------
// dW = H^T . G fused with the SGD update.  The contraction runs over the batch
// (M rows, 32 per MFMA step), so per weight there are only M multiply-adds and
// the kernel is bound by the read-modify-write of the float master weights
// (4 B read, 4 B + 2 B written per weight).
//
// One wavefront owns a 64 (k) x 64 (n) block of W; a workgroup is four such
// blocks side by side.  Lane (c, g) loads the 8 x 4 blocks H[m0+8g ..][k0+4c ..]
// and G[m0+8g ..][n0+4c ..] (8-byte loads), transposes them in registers into
// four A and four B operands of v_mfma_f32_16x16x32_bf16; MFMA (i, j) yields
// rows k0 + 4*rho + i, columns n0 + 4*c + j.  A lane ends up with 16 rows x 4
// consecutive columns, so master weights move as 16-byte vectors, 256
// contiguous bytes per row across the 16 lanes.  The master-weight loads are
// issued before the MFMA phase and complete underneath it.
// ---------------------------------------------------------------------------
struct UpdateArgs {
    uint32_t n;
    uint32_t pad;
    UpdateProblem p[kMaxProblems];
};

constexpr int kUpdK = 64, kUpdN = 256;      // workgroup tile

// Which update problem and tile workgroup `id` owns: lane i holds job i's tile count.
__device__ inline int find_update(const UpdateProblem *p, uint32_t n, uint32_t id, uint32_t *t, uint32_t *kt)
{
    const int lane = threadIdx.x & 63;
    const bool valid = lane < (int)n;
    uint32_t k_tiles = 0, count = 0;
    if (valid) {
        k_tiles = (p[lane].K + kUpdK - 1) / kUpdK;
        count = k_tiles * ((p[lane].N + kUpdN - 1) / kUpdN);
    }
    const uint32_t first = wave_excl_scan_u32(count, nullptr);
    const int job = __builtin_amdgcn_readfirstlane(wave_find_range(first, id, valid));
    *t = id - __shfl(first, job, 64);
    *kt = __shfl(k_tiles, job, 64);
    return job;
}

// Tile t of one job's update (kt = its number of 64-row tiles).
__device__ inline void dw_sgd_tile(const UpdateProblem &p, uint32_t t, uint32_t kt)
{
    const int lane = threadIdx.x & 63, c = lane & 15, g = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t M = p.M, K = p.K, N = p.N;
    const uint32_t k0 = (t % kt) * kUpdK;                  // neighbours share the G columns
    const uint32_t n0 = (t / kt) * kUpdN + 64 * wave;
    const uint32_t ncol = n0 + 4 * c;
    const bool col_ok = ncol < N;
    const uint16_t *H = (const uint16_t *)p.H;
    const uint16_t *G = (const uint16_t *)p.G;

    // master weights of this lane: rows k0 + 16g + 4r + i, columns ncol .. ncol+3
    f32x4 wm[16];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t krow = k0 + 16 * g + 4 * r + i;
            wm[r * 4 + i] = (krow < K && col_ok)
                                ? __builtin_nontemporal_load((const f32x4 *)(p.Wm + (size_t)krow * N + ncol))
                                : f32x4{0.f, 0.f, 0.f, 0.f};
        }

    f32x4 acc[16];      // acc[i * 4 + j][r]
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    const uint32_t kcol = k0 + 4 * c;
    const bool kcol_ok = kcol < K;
    for (uint32_t m0 = 0; m0 < M; m0 += 32) {
        u32x2 h[8], d[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const uint32_t m = m0 + 8 * g + r;
            h[r] = (m < M && kcol_ok) ? *(const u32x2 *)(H + (size_t)m * K + kcol) : u32x2{0u, 0u};
            d[r] = (m < M && col_ok) ? *(const u32x2 *)(G + (size_t)m * N + ncol) : u32x2{0u, 0u};
        }
        u32x4 A[4], B[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t sel = (i & 1) ? 0x07060302u : 0x05040100u;
                A[i][j] = __builtin_amdgcn_perm(h[2 * j + 1][i >> 1], h[2 * j][i >> 1], sel);
                B[i][j] = __builtin_amdgcn_perm(d[2 * j + 1][i >> 1], d[2 * j][i >> 1], sel);
            }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i * 4 + j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                    __builtin_bit_cast(bf16x8, A[i]), __builtin_bit_cast(bf16x8, B[j]), acc[i * 4 + j],
                    0, 0, 0);
    }

    const float lr = p.lr;
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t krow = k0 + 16 * g + 4 * r + i;
            if (krow >= K || !col_ok) continue;
            f32x4 w = wm[r * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j)      // one rounded multiply, one rounded subtract
                w[j] = __fsub_rn(w[j], __fmul_rn(lr, acc[i * 4 + j][r]));
            __builtin_nontemporal_store(w, (f32x4 *)(p.Wm + (size_t)krow * N + ncol));
            u32x2 b;
            b[0] = bf16_pack(w[0], w[1]);
            b[1] = bf16_pack(w[2], w[3]);
            *(u32x2 *)((uint16_t *)p.Wb + (size_t)krow * N + ncol) = b;
        }
}

__global__ __launch_bounds__(256) void grouped_dw_sgd(UpdateArgs a)
{
    uint32_t t, kt;
    const int job = find_update(a.p, a.n, blockIdx.x, &t, &kt);
    dw_sgd_tile(a.p[job], t, kt);
}

hipError_t launch_grouped_dw_sgd(const UpdateProblem *p, uint32_t n, hipStream_t stream,
                                 uint64_t *launches)
{
    for (uint32_t at = 0; at < n; at += kMaxProblems) {
        UpdateArgs a{};
        a.n = std::min(kMaxProblems, n - at);
        uint64_t tiles = 0;
        for (uint32_t i = 0; i < a.n; ++i) {
            a.p[i] = p[at + i];
            tiles += (uint64_t)((a.p[i].K + kUpdK - 1) / kUpdK) * ((a.p[i].N + kUpdN - 1) / kUpdN);
        }
        if (tiles == 0) continue;
        if (tiles > 0x7fffffffull) return hipErrorInvalidValue;
        hipLaunchKernelGGL(grouped_dw_sgd, dim3((uint32_t)tiles), dim3(256), 0, stream, a);
        if (launches) *launches += 1;
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace salus
