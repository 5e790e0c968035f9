// Training-step kernels for gfx950: softmax cross-entropy with its gradient,
// and the fused weight-gradient + SGD update.  (The input-gradient product
// dX = dY . W^T reuses grouped_dense_bf16 with the transposed-weight load path.)
//
// A training iteration is a forward pass, a backward pass and a parameter
// update (Salus paper, Section 2.1); hyper-parameter tuning packs many such
// jobs of one architecture on a GPU (Section 5.2).  All jobs of a round share
// every launch here, as in the forward pass.
#include <algorithm>

#include "device.hpp"
#include "wave.hpp"

namespace salus {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

__device__ inline uint32_t bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

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
// (softmax - onehot) / M, written as bf16 for the backward products.  One
// wavefront per row (a workgroup takes four rows of one job; the job is found
// with the scan + ballot used everywhere else); each row's loss goes to a
// scratch array and a second, tiny kernel adds the rows of a job in order, so
// the result does not depend on how the rows were scheduled.
// ---------------------------------------------------------------------------
struct LossArgs {
    uint32_t n;
    uint32_t pad;
    LossProblem p[kMaxProblems];
};

__global__ __launch_bounds__(256) void softmax_xent_rows(LossArgs a)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool valid = lane < (int)a.n;
    const uint32_t blocks = valid ? (a.p[lane].M + 3) / 4 : 0;
    const uint32_t first = wave_excl_scan_u32(blocks, nullptr);
    const int job = __builtin_amdgcn_readfirstlane(wave_find_range(first, blockIdx.x, valid));
    const LossProblem &p = a.p[job];
    const uint32_t row = (blockIdx.x - __shfl(first, job, 64)) * 4 + wave;
    const uint32_t M = p.M, N = p.N;
    if (row >= M) return;
    const float inv_m = 1.0f / (float)M;
    const float *z = p.logits + (size_t)row * N;
    float zmax = -INFINITY;
    for (uint32_t n = lane; n < N; n += 64) zmax = fmaxf(zmax, z[n]);
    zmax = wave_max(zmax);
    float denom = 0.0f;
    for (uint32_t n = lane; n < N; n += 64) denom += expf(z[n] - zmax);
    denom = wave_sum(denom);
    int label = p.labels[row];
    label = label < 0 ? 0 : (label >= (int)N ? (int)N - 1 : label);    // never read outside the row
    if (lane == 0) p.row_loss[row] = -(z[label] - zmax - logf(denom));
    uint16_t *g = (uint16_t *)p.grad + (size_t)row * N;
    const float inv_d = 1.0f / denom;
    for (uint32_t n = lane; n < N; n += 64) {
        const float prob = expf(z[n] - zmax) * inv_d;
        g[n] = (uint16_t)bf16_rne((prob - ((int)n == label ? 1.0f : 0.0f)) * inv_m);
    }
}

__global__ __launch_bounds__(64) void loss_mean(LossArgs a)
{
    const LossProblem &p = a.p[blockIdx.x];
    if (threadIdx.x != 0) return;
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
        for (uint32_t i = 0; i < a.n; ++i) {
            a.p[i] = p[at + i];
            blocks += (a.p[i].M + 3) / 4;
        }
        if (blocks == 0) continue;
        if (blocks > 0x7fffffffull) return hipErrorInvalidValue;
        hipLaunchKernelGGL(softmax_xent_rows, dim3((uint32_t)blocks), dim3(256), 0, stream, a);
        hipLaunchKernelGGL(loss_mean, dim3(a.n), dim3(64), 0, stream, a);
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

__global__ __launch_bounds__(256) void grouped_dw_sgd(UpdateArgs a)
{
    const int lane = threadIdx.x & 63, c = lane & 15, g = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // job lookup: lane i holds job i's tile count
    const bool valid = lane < (int)a.n;
    uint32_t k_tiles = 0, count = 0;
    if (valid) {
        k_tiles = (a.p[lane].K + kUpdK - 1) / kUpdK;
        count = k_tiles * ((a.p[lane].N + kUpdN - 1) / kUpdN);
    }
    const uint32_t first = wave_excl_scan_u32(count, nullptr);
    const int job = __builtin_amdgcn_readfirstlane(wave_find_range(first, blockIdx.x, valid));
    const uint32_t t = blockIdx.x - __shfl(first, job, 64);
    const uint32_t kt = __shfl(k_tiles, job, 64);
    const UpdateProblem &p = a.p[job];
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
            b[0] = bf16_rne(w[0]) | (bf16_rne(w[1]) << 16);
            b[1] = bf16_rne(w[2]) | (bf16_rne(w[3]) << 16);
            *(u32x2 *)((uint16_t *)p.Wb + (size_t)krow * N + ncol) = b;
        }
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
