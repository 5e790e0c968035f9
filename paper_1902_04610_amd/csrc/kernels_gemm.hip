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

#include "dense_tile.hpp"

namespace salus {

template <int MT, bool TW, bool NT>
__global__ __launch_bounds__(kGemmThreads) void grouped_dense_bf16(GroupArgs a)
{
    __shared__ float lds[reduce_lds_floats<MT * 8>()];
    const Tile tile = find_tile<16 * MT, 128>(a);
    dense_bf16_tile<MT, TW, NT>(a.p[tile.problem], tile, lds);
}

template <int MT>
__global__ __launch_bounds__(kGemmThreads) void grouped_dense_f32(GroupArgs a)
{
    __shared__ float lds[reduce_lds_floats<MT * 4>()];
    const Tile tile = find_tile<16 * MT, 64>(a);
    dense_f32_tile<MT>(a.p[tile.problem], tile, lds);
}

// ---------------------------------------------------------------------------
template <typename Launch>
static hipError_t launch_groups(const Problem *p, uint32_t n, uint32_t tn, uint32_t m_small,
                                uint32_t m_mid, Launch launch, uint64_t *launches)
{
    for (uint32_t at = 0; at < n; at += kMaxProblems) {
        GroupArgs a{};
        a.n = std::min(kMaxProblems, n - at);
        uint32_t max_m = 0;
        for (uint32_t i = 0; i < a.n; ++i) {
            a.p[i] = p[at + i];
            max_m = std::max(max_m, a.p[i].M);
        }
        const int mt = max_m <= m_small ? 1 : max_m <= m_mid ? 2 : 4;
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
    auto launch = [&](int mt, const GroupArgs &a, uint32_t tiles) {
        const dim3 grid(tiles), block(kGemmThreads);
        // mt == 1 means no job has more than 16 rows; with mt == 2 a job above 32
        // rows has several row tiles that read the same weights
        bool one_row_tile = true;
        for (uint32_t i = 0; i < a.n; ++i) one_row_tile = one_row_tile && a.p[i].M <= 16u * mt;
        if (trans_w) {
            if (mt == 1) hipLaunchKernelGGL((grouped_dense_bf16<1, true, true>), grid, block, 0, stream, a);
            else if (one_row_tile) hipLaunchKernelGGL((grouped_dense_bf16<2, true, true>), grid, block, 0, stream, a);
            else hipLaunchKernelGGL((grouped_dense_bf16<2, true, false>), grid, block, 0, stream, a);
        } else {
            if (mt == 1) hipLaunchKernelGGL((grouped_dense_bf16<1, false, true>), grid, block, 0, stream, a);
            else if (one_row_tile) hipLaunchKernelGGL((grouped_dense_bf16<2, false, true>), grid, block, 0, stream, a);
            else hipLaunchKernelGGL((grouped_dense_bf16<2, false, false>), grid, block, 0, stream, a);
        }
    };
    // Row tiles of at most 32 rows: a 64-row tile halves the workgroup count and
    // the occupancy, and measured slower even though W is then read once instead
    // of twice (the second read of neighbouring row tiles hits L2).
    return launch_groups(p, n, 128, 16, 1u << 30, launch, launches);
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
