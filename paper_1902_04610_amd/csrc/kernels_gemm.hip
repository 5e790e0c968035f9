// Grouped dense-layer kernels for gfx950 (MI355X): one launch runs one layer of
// every job scheduled in the round.  This is how "parallelism across lanes"
// (Salus paper, Section 3.3) is executed here: instead of one GPU stream per
// lane, the tiles of all lanes' jobs share one grid, and each workgroup finds
// its job with a wavefront scan over the per-job tile counts.
//
// Shape of the work: per job Y[M x N] = act(X[M x K] . W[K x N]) with M small
// (1..64 rows) and W read straight out of the job's persistent block.  Every
// weight is used once per launch, so the kernel is a weight-streaming kernel:
// W goes HBM -> registers with 16-byte loads (no LDS staging: nothing would be
// reused), each wavefront keeps two k-steps of loads in flight, the 8x8 bf16
// sub-blocks are transposed in registers into MFMA operand order, and the four
// wavefronts of a workgroup split K and combine their partial tiles through LDS.
#include <algorithm>
#include <vector>

#include "dense_tile_n64.hpp"

namespace salus {

template <int MT, bool TW, bool NT>
__global__ __launch_bounds__(kGemmThreads) void grouped_dense_bf16(GroupArgs a)
{
    __shared__ float lds[reduce_lds_floats<MT * 8>()];
    const Tile tile = find_tile<16 * MT, 128>(a);
    const Problem &p = a.p[tile.problem];
    // A job of at most 16 rows takes the one-row-tile path even when the launch holds
    // larger jobs: its second row tile would only load clamped copies of its last row,
    // and activation loads count against the compute unit's memory path like weights do.
    if (MT == 2 && NT && p.M <= 16) dense_bf16_tile<1, TW, NT>(p, tile, lds);
    else dense_bf16_tile<MT, TW, NT>(p, tile, lds);
}

// 64-row tiles of 128 columns for deep layers of jobs with 33 .. 128 rows: every weight passes through a
// compute unit once.  Two workgroups per compute unit (registers capped accordingly), so that one
// workgroup's reduction and epilogue overlap the other's stream.
template <bool NT>
__global__ __launch_bounds__(kGemmThreads, 2) void grouped_dense_bf16_rows64(GroupArgs a)
{
    __shared__ float lds[reduce_lds_floats<32>()];
    const Tile tile = find_tile<64, 128>(a);
    dense_bf16_tile<4, false, NT>(a.p[tile.problem], tile, lds);
}

// Jobs of 33 .. 128 rows that do not go to the LDS-tiled kernel: row tiles of 64
// rows, 64 columns wide (see dense_tile_n64.hpp).
template <bool TW, bool NT>
__global__ __launch_bounds__(kGemmThreads) void grouped_dense_bf16_n64(GroupArgs a)
{
    __shared__ float lds[reduce_lds_floats<16>()];
    const Tile tile = find_tile<64, 64>(a);
    dense_bf16_tile_n64<4, TW, NT>(a.p[tile.problem], tile, lds);
}

template <int MT>
__global__ __launch_bounds__(kGemmThreads) void grouped_dense_f32(GroupArgs a)
{
    __shared__ float lds[reduce_lds_floats<MT * 4>()];
    const Tile tile = find_tile<16 * MT, 64>(a);
    dense_f32_tile<MT>(a.p[tile.problem], tile, lds);
}

// ---------------------------------------------------------------------------
// force_mt != 0: row tiles of 16 * force_mt rows whatever the jobs' sizes
template <typename Launch>
static hipError_t launch_groups(const Problem *p, uint32_t n, uint32_t tn, uint32_t m_small,
                                uint32_t m_mid, Launch launch, uint64_t *launches, int force_mt = 0)
{
    for (uint32_t at = 0; at < n; at += kMaxProblems) {
        GroupArgs a{};
        a.n = std::min(kMaxProblems, n - at);
        uint32_t max_m = 0;
        for (uint32_t i = 0; i < a.n; ++i) {
            a.p[i] = p[at + i];
            max_m = std::max(max_m, a.p[i].M);
        }
        const int mt = force_mt ? force_mt : max_m <= m_small ? 1 : max_m <= m_mid ? 2 : 4;
        const uint32_t tm = 16u * mt;
        uint64_t tiles = 0;
        for (uint32_t i = 0; i < a.n; ++i)
            tiles += (uint64_t)((a.p[i].M + tm - 1) / tm) * ((a.p[i].N + tn - 1) / tn);
        if (tiles == 0) continue;
        if (tiles > 0x7fffffffull) return hipErrorInvalidValue;
        launch(mt, a, (uint32_t)tiles);
        if (launches) *launches += 1;
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// Rows per job from which the LDS-tiled kernel is used: always from 128 rows; from
// 65 rows (where the streaming kernel needs a third row tile) if the jobs routed
// there make up at least one workgroup per CU (256).  Up to 64 rows the
// streaming kernel's two row tiles run side by side and the second one finds the
// weights in L2, which measured faster than a half-empty 128-row tile.
constexpr uint32_t kTiledAlways = 128, kTiledMaybe = 65;
constexpr uint64_t kTiledMinGrid = 256;
constexpr uint64_t kFullGrid = 256;      // one workgroup per compute unit
constexpr uint32_t kDeepK = 1024;

hipError_t launch_grouped_bf16(const Problem *p, uint32_t n, bool trans_w, hipStream_t stream,
                               uint64_t *launches)
{
    // Jobs with many rows reuse every weight often enough to pay for LDS staging:
    // they go to the tiled kernel, the rest of the round to the streaming kernel.
    if (!trans_w) {
        uint64_t grid = 0;
        for (uint32_t i = 0; i < n; ++i)
            if (p[i].M >= kTiledMaybe && tiled_shape_ok(p[i])) grid += tiled_tiles(p[i]);
        const uint32_t min_m = grid >= kTiledMinGrid ? kTiledMaybe : kTiledAlways;
        std::vector<Problem> tiled, streamed;
        for (uint32_t i = 0; i < n; ++i)
            (p[i].M >= min_m && tiled_shape_ok(p[i]) ? tiled : streamed).push_back(p[i]);
        if (!tiled.empty()) {
            hipError_t e = launch_grouped_bf16_tiled(tiled.data(), (uint32_t)tiled.size(), stream, launches);
            if (e != hipSuccess || streamed.empty()) return e;
            return launch_grouped_bf16(streamed.data(), (uint32_t)streamed.size(), false, stream, launches);
        }
    }
    // Up to 32 rows: one row tile of 16 or 32 rows per job, 128 columns, every weight
    // read once (non-temporal).  33 .. 128 rows (those the tiled kernel did not take):
    // when 64-row tiles of 128 columns would not even make one workgroup per compute
    // unit (a few training jobs, say), row tiles of 64 rows and 64 columns: twice the
    // workgroups, and the weights pass through a compute unit's memory path once per
    // 64 rows (2048 x 2048 layers of 8 jobs at 64 rows: 21.0 us against 22.7 us
    // forward, 21.4 against 28.2 us for the input gradient, whose rows are then read
    // in whole cache lines).  With enough jobs to fill the chip: layers at least 1024 deep
    // get one 64-row tile of 128 columns per workgroup, so that every weight passes through
    // a compute unit once, with registers capped for two workgroups per compute unit (64
    // models of the inference workload at 48 / 64 rows: 0.250 / 0.270 ms per round against
    // 0.287 / 0.300 ms with two 32-row tiles, the second of which reads the weights from L2;
    // the same 64-row tile uncapped, one workgroup per compute unit, had been 5 % slower
    // than the two 32-row tiles on 1024-deep layers: nothing then overlaps a workgroup's
    // reduction and epilogue); shallower layers, transposed weights and jobs above 128 rows
    // keep 32-row tiles of 128 columns.
    std::vector<Problem> small, mid, large;
    for (uint32_t i = 0; i < n; ++i)
        (p[i].M <= 32 ? small : p[i].M <= 128 ? mid : large).push_back(p[i]);
    auto launch_wide = [&](int mt, const GroupArgs &a, uint32_t tiles) {
        const dim3 grid(tiles), block(kGemmThreads);
        bool one_row_tile = true;      // else several row tiles read the same weights: plain loads, L2 serves the others
        for (uint32_t i = 0; i < a.n; ++i) one_row_tile = one_row_tile && a.p[i].M <= 16u * mt;
#define SALUS_WIDE(MT_)                                                                                        \
        do {                                                                                                    \
            if (trans_w && one_row_tile) hipLaunchKernelGGL((grouped_dense_bf16<MT_, true, true>), grid, block, 0, stream, a);   \
            else if (trans_w) hipLaunchKernelGGL((grouped_dense_bf16<MT_, true, false>), grid, block, 0, stream, a);            \
            else if (one_row_tile) hipLaunchKernelGGL((grouped_dense_bf16<MT_, false, true>), grid, block, 0, stream, a);       \
            else hipLaunchKernelGGL((grouped_dense_bf16<MT_, false, false>), grid, block, 0, stream, a);                        \
        } while (0)
        if (mt == 4) {      // forward only (the launcher never asks for it with transposed weights)
            if (one_row_tile) hipLaunchKernelGGL((grouped_dense_bf16_rows64<true>), grid, block, 0, stream, a);
            else hipLaunchKernelGGL((grouped_dense_bf16_rows64<false>), grid, block, 0, stream, a);
            return;
        }
        if (mt == 1) SALUS_WIDE(1);
        else SALUS_WIDE(2);
#undef SALUS_WIDE
    };
    auto launch_n64 = [&](int, const GroupArgs &a, uint32_t tiles) {
        const dim3 grid(tiles), block(kGemmThreads);
        bool one_row_tile = true;
        for (uint32_t i = 0; i < a.n; ++i) one_row_tile = one_row_tile && a.p[i].M <= 64u;
        if (trans_w && one_row_tile) hipLaunchKernelGGL((grouped_dense_bf16_n64<true, true>), grid, block, 0, stream, a);
        else if (trans_w) hipLaunchKernelGGL((grouped_dense_bf16_n64<true, false>), grid, block, 0, stream, a);
        else if (one_row_tile) hipLaunchKernelGGL((grouped_dense_bf16_n64<false, true>), grid, block, 0, stream, a);
        else hipLaunchKernelGGL((grouped_dense_bf16_n64<false, false>), grid, block, 0, stream, a);
    };
    if (!small.empty())
        if (hipError_t e = launch_groups(small.data(), (uint32_t)small.size(), 128, 16, 32, launch_wide, launches)) return e;
    if (!mid.empty()) {
        uint64_t wide_tiles = 0;
        for (const Problem &q : mid) wide_tiles += (uint64_t)((q.M + 63) / 64) * ((q.N + 127) / 128);
        hipError_t e = hipSuccess;
        if (wide_tiles < kFullGrid) {
            e = launch_groups(mid.data(), (uint32_t)mid.size(), 64, 0, 0, launch_n64, launches, 4);
        } else {
            std::vector<Problem> deep, shallow;
            for (const Problem &q : mid) (!trans_w && q.K >= kDeepK ? deep : shallow).push_back(q);
            if (!shallow.empty())
                e = launch_groups(shallow.data(), (uint32_t)shallow.size(), 128, 0, 0, launch_wide, launches, 2);
            if (e == hipSuccess && !deep.empty())
                e = launch_groups(deep.data(), (uint32_t)deep.size(), 128, 0, 0, launch_wide, launches, 4);
        }
        if (e != hipSuccess) return e;
    }
    if (!large.empty())
        if (hipError_t e = launch_groups(large.data(), (uint32_t)large.size(), 128, 0, 0, launch_wide, launches, 2)) return e;
    return hipSuccess;
}

hipError_t launch_grouped_f32(const Problem *p, uint32_t n, hipStream_t stream, uint64_t *launches)
{
    auto launch = [&](int mt, const GroupArgs &a, uint32_t tiles) {
        if (mt == 1)
            hipLaunchKernelGGL(grouped_dense_f32<1>, dim3(tiles), dim3(kGemmThreads), 0, stream, a);
        else if (mt == 2)
            hipLaunchKernelGGL(grouped_dense_f32<2>, dim3(tiles), dim3(kGemmThreads), 0, stream, a);
        else
            hipLaunchKernelGGL(grouped_dense_f32<4>, dim3(tiles), dim3(kGemmThreads), 0, stream, a);
    };
    return launch_groups(p, n, 64, 16, 32, launch, launches);
}

}  // namespace salus
