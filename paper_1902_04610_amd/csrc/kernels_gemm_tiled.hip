// Grouped dense layer for jobs that bring many rows (M >= 128, or more than 64
// when the round holds enough of them to give every CU a tile): the
// compute-bound counterpart of the weight-streaming kernel.  Same contract (one
// launch runs one layer of every scheduled job, Salus paper, Section 3.3), but
// here a weight is used by 128 or 256 rows per workgroup, so operands are staged
// through LDS.
//
// Workgroup tile BM x 256 (BM = 256 for jobs from 192 rows, else 128), k-slab 64,
// eight wavefronts (4 x 2 of 64 x 128, or 2 x 4 of 64 x 64), v_mfma_f32_32x32x16_bf16.
//   HBM -> registers : 16-byte loads, issued two slabs ahead of the multiply
//   registers -> LDS : X rows as they are; W blocks of 4 k x 8 n are transposed in
//                      registers first, so that both operands sit in LDS as
//                      [row or column][64 k-values] = 128 bytes per line
//   LDS -> registers : one ds_read_b128 per 32x16 operand fragment
// LDS holds two slabs: the slab after the one being multiplied is written while
// it is multiplied - a quarter of the writes after each quarter of the MFMAs, so
// that they issue while the matrix pipe works through its queue - and the one
// after that is on its way from memory; one barrier per slab.  One workgroup
// fills a CU (registers at BM = 256, LDS at BM = 128), so this overlap has to
// come from inside it.  Per multiply-add the 256-row tile moves a third less
// through L2 than the 128-row one ((256 + 256) / (256 * 256) against
// (128 + 256) / (128 * 256) operand bytes).
// The 16-byte slot of k-chunk c in line r is c ^ swz(r), swz(r) = (r ^ r/8) % 8.
// Fragment reads touch 32 consecutive lines at one k-chunk, the transposed W
// writes touch lines 8 apart at one k-chunk, X writes fill whole lines: with
// this swizzle each of them spreads every 8 lanes that the LDS serves together
// over all 8 slots of the 128-byte bank row (measured: no bank conflicts).
#include <algorithm>
#include <vector>

#include "group.hpp"

namespace salus {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kBM = 128, kBN = 256, kBK = 64;
constexpr int kLine = kBK * 2;                 // bytes per LDS line

__device__ inline uint32_t swz(uint32_t line) { return (line ^ (line >> 3)) & 7u; }

// Tiles of one job in bands of 8 row tiles, column tiles inside a band: the 64
// tiles an XCD runs at a time then share 8 slabs of X and 8 slabs of W in its L2.
template <int BM, int BN>
__device__ inline Tile find_tile_banded(const GroupArgs &a, uint32_t tile_id)
{
    const int lane = threadIdx.x & 63;
    const bool valid = lane < (int)a.n;
    uint32_t row_tiles = 0, col_tiles = 0;
    if (valid) {
        row_tiles = (a.p[lane].M + BM - 1) / BM;
        col_tiles = (a.p[lane].N + BN - 1) / BN;
    }
    const uint32_t first = wave_excl_scan_u32(row_tiles * col_tiles, nullptr);
    // the grid is a multiple of 8, so a workgroup's tiles all map to its own XCD's range
    const uint32_t id = xcd_remap(tile_id, a.tiles);
    const int g = wave_find_range(first, id, valid);
    const uint32_t t = id - __shfl(first, g, 64);
    const uint32_t rt = __shfl(row_tiles, g, 64), ct = __shfl(col_tiles, g, 64);
    const uint32_t band = t / (8u * ct), local = t - band * 8u * ct;
    const uint32_t rows = min(8u, rt - band * 8u);
    Tile tile;
    tile.problem = __builtin_amdgcn_readfirstlane(g);
    tile.m0 = (band * 8u + local % rows) * BM;
    tile.n0 = (local / rows) * BN;
    return tile;
}

template <int ACT, int FM, int FN>
__device__ inline void store_tile(const f32x16 (&acc)[FM][FN], const Problem &p, const Tile &tile,
                                  uint32_t wm, uint32_t wn, uint32_t fl, uint32_t fh)
{
    const uint32_t M = p.M, N = p.N;
    const bool out_bf16 = (p.flags & kOutBf16) != 0, mask = (p.flags & kMaskPositive) != 0;
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        const uint32_t col = tile.n0 + wn * (32u * FN) + 32u * j + fl;
        if (col >= N) continue;
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            const uint32_t row0 = tile.m0 + wm * (32u * FM) + 32u * i + 4u * fh;
            float v[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float z = acc[i][j][r];
                v[r] = ACT == 1 ? fmaxf(z, 0.0f) : ACT == 2 ? gelu_fast(z) : z;
            }
            if (mask) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const uint32_t row = row0 + 8u * (r >> 2) + (r & 3);
                    if (row >= M) continue;
                    const uint32_t bits = ((const uint16_t *)p.aux)[(size_t)row * N + col];
                    if ((bits & 0x8000u) || !(bits & 0x7fffu)) v[r] = 0.0f;
                }
            }
            if (out_bf16) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const uint32_t row = row0 + 8u * (r >> 2) + (r & 3);
                    if (row < M) ((uint16_t *)p.Y)[(size_t)row * N + col] = (uint16_t)bf16_bits(v[r]);
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const uint32_t row = row0 + 8u * (r >> 2) + (r & 3);
                    if (row < M) ((float *)p.Y)[(size_t)row * N + col] = v[r];
                }
            }
        }
    }
}

// Epilogue of a tile that lies wholly inside its matrix (and whose matrix is
// below 4 GiB): no bounds tests, 32-bit byte offsets from the uniform base
// pointer, activation and output type fixed at compile time.  This is the
// common case; the general routine above costs about twice the instructions.
template <int ACT, bool BF16, int FM, int FN>
__device__ inline void store_tile_full(const f32x16 (&acc)[FM][FN], const Problem &p, const Tile &tile,
                                       uint32_t wm, uint32_t wn, uint32_t fl, uint32_t fh)
{
    constexpr uint32_t esz = BF16 ? 2u : 4u;
    const uint32_t row_bytes = p.N * esz;
    char *Y = (char *)p.Y;
#pragma unroll
    for (int j = 0; j < FN; ++j) {
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            const uint32_t row0 = tile.m0 + wm * (32u * FM) + 32u * i + 4u * fh;
            const uint32_t col = tile.n0 + wn * (32u * FN) + 32u * j + fl;
            const uint32_t off0 = row0 * row_bytes + col * esz;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float z = acc[i][j][r];
                const float v = ACT == 1 ? fmaxf(z, 0.0f) : ACT == 2 ? gelu_fast(z) : z;
                const uint32_t off = off0 + (8u * (r >> 2) + (r & 3)) * row_bytes;
                if (BF16) *(uint16_t *)(Y + off) = (uint16_t)bf16_bits(v);
                else *(float *)(Y + off) = v;
            }
        }
    }
}

// Requires K % 64 == 0 and N % 8 == 0 (the launcher routes other shapes to the
// streaming kernel).  Rows >= M and columns >= N are loaded from clamped
// addresses and never stored.  A thread owns BM / 64 16-byte k-chunks of X (rows
// 64 apart) and a block of 4 k x 8 columns of W, which it transposes into eight
// 8-byte half-chunks.
constexpr int kBM2 = 256, kThreads2 = 512;

// BM2 = 256: wavefronts 4 x 2, each 64 x 128.  BM2 = 128: 2 x 4, each 64 x 64.
// The grid is one workgroup per CU; workgroup b runs tiles b, b + grid, ... and
// requests the first slab of its next tile before the epilogue of the current
// one, so that neither that latency nor a workgroup launch sits between tiles.
template <int BM2>
__global__ __launch_bounds__(kThreads2) void grouped_dense_bf16_tiled(GroupArgs a)
{
    constexpr uint32_t kStageBytes = (BM2 + kBN) * kLine;      // 64 KB or 48 KB
    constexpr int WN = BM2 == 256 ? 2 : 4, FN = kBN / (32 * WN), XR = BM2 / 64;
    __shared__ __attribute__((aligned(128))) unsigned char smem[2 * kStageBytes];
    const uint32_t t = threadIdx.x, lane = t & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const uint32_t wm = wave / WN, wn = wave % WN;

    // X: k-chunk ca of rows ra, ra+64, ... (lines 64 apart share their swizzle)
    const uint32_t ca = t & 7u, ra = t >> 3;
    const uint32_t xoff = ra * kLine + ((ca ^ swz(ra)) << 4);
    // W: rows 4*kq .. 4*kq+3 of the slab, columns 8*nb .. 8*nb+7
    const uint32_t kq = (lane >> 3) + 8u * (wave >> 2), nb = (lane & 7u) + 8u * (wave & 3u);
    uint32_t woff[8];      // byte offset of this thread's half-chunk in column line 8*nb + i
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint32_t line = 8u * nb + i;
        woff[i] = (BM2 + line) * kLine + (((kq >> 1) ^ swz(line)) << 4) + 8u * (kq & 1u);
    }

    struct Source {           // where this thread's part of a tile's operands comes from
        Tile tile;
        const uint16_t *x[XR];
        const uint16_t *w;
        uint32_t wpitch;
    };
    auto locate = [&](uint32_t id) {
        Source src;
        src.tile = find_tile_banded<BM2, kBN>(a, id);
        const Problem &p = a.p[src.tile.problem];
        const uint32_t M = p.M, K = p.K, N = p.N;
        const uint16_t *W = (const uint16_t *)p.W;
        const uint16_t *X = (const uint16_t *)p.X;
#pragma unroll
        for (int i = 0; i < XR; ++i) {
            const uint32_t row = src.tile.m0 + ra + 64u * i;
            src.x[i] = X + (size_t)(row < M ? row : M - 1) * K + 8u * ca;
        }
        const uint32_t ncol = src.tile.n0 + 8u * nb, ncol_c = ncol < N ? ncol : 0u;
        const bool strip = (p.flags & kStripW) != 0;
        src.wpitch = strip ? 128u : N;
        src.w = strip ? W + (size_t)(ncol_c & ~127u) * K + (4u * kq) * 128u + (ncol_c & 127u)
                      : W + (size_t)(4u * kq) * N + ncol_c;
        return src;
    };

    u32x4 xr[XR], wr[4];
    auto load_slab = [&](const Source &src, uint32_t k0) {
#pragma unroll
        for (int i = 0; i < XR; ++i) xr[i] = *(const u32x4 *)(src.x[i] + k0);
#pragma unroll
        for (int r = 0; r < 4; ++r) wr[r] = *(const u32x4 *)(src.w + (size_t)(k0 + r) * src.wpitch);
    };
    auto store_x = [&](uint32_t stage) {
        unsigned char *base = smem + stage;
#pragma unroll
        for (int i = 0; i < XR; ++i) *(u32x4 *)(base + xoff + 64 * i * kLine) = xr[i];
    };
    auto store_w = [&](uint32_t stage, int first) {      // columns first .. first+3 of the block
        unsigned char *base = smem + stage;
#pragma unroll
        for (int i = first; i < first + 4; ++i) {
            u32x2 b;       // column i of the block: dword j = (k 2j, k 2j+1)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                b[j] = __builtin_amdgcn_perm(wr[2 * j + 1][i >> 1], wr[2 * j][i >> 1],
                                             (i & 1) ? 0x07060302u : 0x05040100u);
            *(u32x2 *)(base + woff[i]) = b;
        }
    };

    const uint32_t fl = lane & 31u, fh = lane >> 5, fs = swz(fl);
    const uint32_t afrag = (wm * 64u + fl) * kLine;
    const uint32_t bfrag = (BM2 + wn * (32u * FN) + fl) * kLine;

    f32x16 acc[2][FN];
    auto multiply = [&](const unsigned char *base, uint32_t ks) {
        const uint32_t off = ((2u * ks + fh) ^ fs) << 4, off_odd = off ^ 64u;
        bf16x8 av[2], bv[FN];
#pragma unroll
        for (int i = 0; i < 2; ++i) av[i] = *(const bf16x8 *)(base + afrag + 32 * i * kLine + (i & 1 ? off_odd : off));
#pragma unroll
        for (int j = 0; j < FN; ++j) bv[j] = *(const bf16x8 *)(base + bfrag + 32 * j * kLine + (j & 1 ? off_odd : off));
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[i], bv[j], acc[i][j], 0, 0, 0);
    };

    const uint32_t tiles = a.tiles;
    uint32_t id = blockIdx.x;
    Source src = locate(id);
    load_slab(src, 0);
    for (;;) {
        const Problem &p = a.p[src.tile.problem];
        const uint32_t M = p.M, N = p.N, slabs = p.K / kBK;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

        // Slab s is multiplied out of one half of LDS while slab s+1 (already in
        // registers) is written to the other half, a piece after each quarter of the
        // multiplies so that the writes issue while the matrix pipe works through
        // its queue, and slab s+2 is requested from memory.  The last slab has
        // nothing to stage; the load past the end re-reads the last slab instead of
        // branching.
        uint32_t stage = 0;
        __syncthreads();                     // the previous tile's last slab has been read
        store_x(0);
        store_w(0, 0);
        store_w(0, 4);
        load_slab(src, slabs > 1 ? kBK : 0);
        __syncthreads();
        for (uint32_t s = 0; s + 1 < slabs; ++s) {
            const unsigned char *base = smem + stage;
            const uint32_t other = stage ^ kStageBytes;      // everyone left it at the last barrier
            multiply(base, 0);
            store_x(other);
            multiply(base, 1);
            store_w(other, 0);
            multiply(base, 2);
            store_w(other, 4);
            multiply(base, 3);
            load_slab(src, (s + 2 < slabs ? s + 2 : slabs - 1) * kBK);
            __syncthreads();
            stage = other;
        }
        {
            const unsigned char *base = smem + stage;
#pragma unroll
            for (uint32_t ks = 0; ks < 4; ++ks) multiply(base, ks);
        }

        // the next tile's first slab travels while this tile's epilogue runs
        const Tile tile = src.tile;
        const uint32_t next = id + gridDim.x;
        const bool more = next < tiles;
        if (more) {
            src = locate(next);
            load_slab(src, 0);
        }

        const uint32_t act = p.flags & 0xffu;
        const bool full = tile.m0 + BM2 <= M && tile.n0 + kBN <= N && (uint64_t)M * N < (1ull << 30) &&
                          !(p.flags & kMaskPositive);
        if (full && (p.flags & kOutBf16)) {
            if (act == 1) store_tile_full<1, true, 2, FN>(acc, p, tile, wm, wn, fl, fh);
            else if (act == 2) store_tile_full<2, true, 2, FN>(acc, p, tile, wm, wn, fl, fh);
            else store_tile_full<0, true, 2, FN>(acc, p, tile, wm, wn, fl, fh);
        } else if (full) {
            if (act == 1) store_tile_full<1, false, 2, FN>(acc, p, tile, wm, wn, fl, fh);
            else if (act == 2) store_tile_full<2, false, 2, FN>(acc, p, tile, wm, wn, fl, fh);
            else store_tile_full<0, false, 2, FN>(acc, p, tile, wm, wn, fl, fh);
        } else if (act == 1) store_tile<1, 2, FN>(acc, p, tile, wm, wn, fl, fh);
        else if (act == 2) store_tile<2, 2, FN>(acc, p, tile, wm, wn, fl, fh);
        else store_tile<0, 2, FN>(acc, p, tile, wm, wn, fl, fh);
        if (!more) break;
        id = next;
    }
}

bool tiled_shape_ok(const Problem &p) { return p.K != 0 && p.K % kBK == 0 && p.N % 8 == 0; }

uint64_t tiled_tiles(const Problem &p)
{
    return (uint64_t)((p.M + kBM - 1) / kBM) * ((p.N + kBN - 1) / kBN);
}

// Jobs of at least this many rows take the 256-row tile (at most a quarter of
// their last row tile is padding); smaller ones the 128-row tile.
constexpr uint32_t kTiled256MinM = 192;

static uint32_t resident_grid()
{
    static uint32_t cached = 0;
    if (cached) return cached;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 8)
        cus = 256;
    cached = (uint32_t)cus & ~7u;
    return cached;
}

template <int BM, typename Kernel>
static hipError_t launch_tiled(Kernel kernel, int threads, const std::vector<Problem> &p, hipStream_t stream,
                               uint64_t *launches)
{
    const uint32_t n = (uint32_t)p.size();
    for (uint32_t at = 0; at < n; at += kMaxProblems) {
        GroupArgs a{};
        a.n = std::min(kMaxProblems, n - at);
        uint64_t tiles = 0;
        for (uint32_t i = 0; i < a.n; ++i) {
            a.p[i] = p[at + i];
            tiles += (uint64_t)((a.p[i].M + BM - 1) / BM) * ((a.p[i].N + kBN - 1) / kBN);
        }
        if (tiles == 0) continue;
        if (tiles > 0x7fffffffull) return hipErrorInvalidValue;
        a.tiles = (uint32_t)tiles;
        // one workgroup per CU (it fills the CU); a multiple of 8 so that the
        // workgroups of an XCD keep to that XCD's range of tiles
        const uint32_t grid = (uint32_t)std::min<uint64_t>(tiles, resident_grid());
        hipLaunchKernelGGL(kernel, dim3(grid), dim3(threads), 0, stream, a);
        if (launches) *launches += 1;
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// ---------------------------------------------------------------------------
// Calibration: the multiply of grouped_dense_bf16_tiled<256> without its memory
// traffic.  One workgroup of eight wavefronts per CU runs `slabs` times the 32
// MFMAs per wavefront of a 256 x 256 x 64 slab, either on fragments read once
// (lds == 0: what the matrix pipes sustain) or on fragments read from LDS for
// every k-step with one barrier per slab (lds != 0: the tiled kernel's multiply
// and LDS reads, nothing else).  Operands are nonzero (a pattern of small
// integers and fractions): the clock a matrix-bound kernel runs at depends on
// what the multipliers toggle.  Wavefront 0 of workgroup 0 reports the shader
// clocks and the 100 MHz ticks its loop took, so the clock under this load can
// be read off: out[0] = s_memtime difference, out[1] = wall-clock difference.
template <bool LDS>
__global__ __launch_bounds__(kThreads2) void mfma_rate(uint64_t *out, uint32_t slabs)
{
    constexpr int BM = 256, FN = 4;
    __shared__ __attribute__((aligned(128))) unsigned char smem[2 * (BM + kBN) * kLine];
    for (uint32_t i = threadIdx.x; i < 2 * (BM + kBN) * kLine / 4; i += kThreads2) {
        const float a = 0.0625f * (float)((i * 7u) & 63u) - 2.0f, b = 0.03125f * (float)((i * 13u) & 127u) - 2.0f;
        ((uint32_t *)smem)[i] = bf16_pack(a, b);
    }
    __syncthreads();
    const uint32_t t = threadIdx.x, lane = t & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const uint32_t wm = wave >> 1, wn = wave & 1u;
    const uint32_t fl = lane & 31u, fh = lane >> 5, fs = swz(fl);
    const uint32_t afrag = (wm * 64u + fl) * kLine, bfrag = (BM + wn * 128u + fl) * kLine;
    f32x16 acc[2][FN];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    bf16x8 av[2], bv[FN];
    auto read = [&](const unsigned char *base, uint32_t ks) {
        const uint32_t off = ((2u * ks + fh) ^ fs) << 4, off_odd = off ^ 64u;
#pragma unroll
        for (int i = 0; i < 2; ++i) av[i] = *(const bf16x8 *)(base + afrag + 32 * i * kLine + (i & 1 ? off_odd : off));
#pragma unroll
        for (int j = 0; j < FN; ++j) bv[j] = *(const bf16x8 *)(base + bfrag + 32 * j * kLine + (j & 1 ? off_odd : off));
    };
    if (!LDS) read(smem, 0);
    const uint64_t c0 = __builtin_readcyclecounter(), w0 = wall_clock64();
    uint32_t stage = 0;
    for (uint32_t s = 0; s < slabs; ++s) {
#pragma unroll
        for (uint32_t ks = 0; ks < 4; ++ks) {
            if (LDS) read(smem + stage, ks);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[i], bv[j], acc[i][j], 0, 0, 0);
        }
        if (LDS) __syncthreads();
        stage ^= (BM + kBN) * kLine;
    }
    const uint64_t c1 = __builtin_readcyclecounter(), w1 = wall_clock64();
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) sum += acc[i][j][r];
    if (blockIdx.x == 0 && t == 0) {
        out[0] = c1 - c0;
        out[1] = w1 - w0;
    }
    if (sum == 1.2345f) out[2] = 1;        // keeps the multiplies
}

// flop: what the launch computes (2 * 256 * 256 * 64 per slab and workgroup)
hipError_t launch_mfma_rate(uint64_t *dev_out, uint32_t slabs, bool lds, hipStream_t stream, uint64_t *flop)
{
    const uint32_t grid = resident_grid();
    if (lds) hipLaunchKernelGGL(mfma_rate<true>, dim3(grid), dim3(kThreads2), 0, stream, dev_out, slabs);
    else hipLaunchKernelGGL(mfma_rate<false>, dim3(grid), dim3(kThreads2), 0, stream, dev_out, slabs);
    if (flop) *flop = 2ull * 256 * 256 * 64 * slabs * grid;
    return hipGetLastError();
}

hipError_t launch_grouped_bf16_tiled(const Problem *p, uint32_t n, hipStream_t stream, uint64_t *launches)
{
    std::vector<Problem> big, small;
    for (uint32_t i = 0; i < n; ++i) {
        if (!tiled_shape_ok(p[i])) return hipErrorInvalidValue;
        (p[i].M >= kTiled256MinM ? big : small).push_back(p[i]);
    }
    hipError_t e = launch_tiled<kBM2>(grouped_dense_bf16_tiled<kBM2>, kThreads2, big, stream, launches);
    if (e != hipSuccess) return e;
    return launch_tiled<kBM>(grouped_dense_bf16_tiled<kBM>, kThreads2, small, stream, launches);
}

}  // namespace salus
