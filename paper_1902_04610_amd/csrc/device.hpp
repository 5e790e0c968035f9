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
constexpr uint32_t kCopyChunk = 8 * 1024;   // bytes one workgroup moves per grid-stride step

// Copies n mutually independent segments (no destination may overlap another
// segment's source); more than kMaxSeg segments are split over launches.
hipError_t launch_copy(const CopySeg *segs, uint32_t n, hipStream_t stream);

// Device state of the in-place slide kernel: one progress counter per resident
// workgroup and a failure word (16 KB of device memory, allocated once).
constexpr uint32_t kSlideMaxGrid = 4032;
struct SlideState {
    uint32_t *progress = nullptr;   // kSlideMaxGrid counters
    uint32_t *failed = nullptr;     // set to 1 by a workgroup whose bounded wait ran out
    uint32_t max_grid = 0;          // resident workgroups a launch may use (found at the first launch)
    uint32_t spin_limit = 1u << 22; // polls (a microsecond or two each) before a wait gives up: seconds
};
hipError_t slide_state_create(SlideState *st);
void slide_state_destroy(SlideState *st);
hipError_t slide_state_failed(SlideState *st, hipStream_t stream, uint32_t *out);

// memmove toward lower addresses inside one allocation: moves in ascending order,
// dst < src, any overlap of a move with itself.  Every byte is read once and
// written once; nothing outside the moved ranges is touched.
hipError_t launch_slide(char *base, const uint64_t *src, const uint64_t *dst, const uint64_t *len,
                        uint32_t n, SlideState *st, hipStream_t stream, uint64_t *launches);

hipError_t launch_scan_u64(const uint64_t *dev_in, uint32_t n, uint64_t *dev_out, hipStream_t s);
hipError_t launch_fill_pattern(void *dev, uint64_t nbytes, uint64_t seed, hipStream_t s);
// Calibration: a kernel that only loads (nbytes a multiple of 4096, sink 16 device bytes).
hipError_t launch_read_only(const void *dev, uint64_t nbytes, void *sink, hipStream_t s);
hipError_t launch_check_pattern(const void *dev, uint64_t nbytes, uint64_t seed,
                                unsigned long long *dev_bad, hipStream_t s);

// ---- grouped GEMM -----------------------------------------------------------
struct Problem {
    const void *W;       // K x N row-major; with kTransW: N x K row-major (Y = X . W^T)
    const void *X;       // M x K row-major
    void *Y;             // M x N row-major
    const void *aux;     // kMaskPositive: M x N bf16, Y is zeroed where aux <= 0
    uint32_t M, K, N;
    uint32_t flags;      // bits 0-7 activation, then the bits below
};
constexpr uint32_t kMaxProblems = 64;       // problems per launch (one per wavefront lane)
constexpr uint32_t kOutBf16 = 1u << 8;      // store Y as bf16 (round to nearest even)
constexpr uint32_t kMaskPositive = 1u << 9; // multiply Y by [aux > 0] (ReLU derivative)
// Hidden activations of jobs with at most 32 rows are kept in the order the MFMA
// A operand wants them, so that a wavefront's activation load is one contiguous
// kilobyte: 16-byte unit (k-step s, row tile t, k-group g, row c) at index
// ((s * T + t) * 4 + g) * 16 + c, T = ceil(M / 16), holds H[16 t + c][32 s + 8 g .. + 8].
constexpr uint32_t kInBlocked = 1u << 11;   // X is in that order
constexpr uint32_t kOutBlocked = 1u << 12;  // Y (bf16) is written in that order
constexpr uint32_t kBlockedMaxM = 32;
constexpr uint32_t kStripW = 1u << 10;      // W is stored in strips of 128 columns: (k, n) at (n/128 * K + k) * 128 + n % 128

// One launch (or several when n > kMaxProblems): Y_g = act(X_g . W_g) for all g.
hipError_t launch_grouped_bf16(const Problem *p, uint32_t n, bool trans_w, hipStream_t stream,
                               uint64_t *launches);
// Jobs with many rows: LDS-tiled compute-bound kernel (128 x 256 tiles, 256 x 256 from 192 rows).
// tiled_shape_ok says whether a problem may go there (K % 64 == 0, N % 8 == 0),
// tiled_tiles how many workgroups it would occupy.
bool tiled_shape_ok(const Problem &p);
uint64_t tiled_tiles(const Problem &p);
hipError_t launch_grouped_bf16_tiled(const Problem *p, uint32_t n, hipStream_t stream,
                                     uint64_t *launches);
// Calibration: the tiled kernel's multiply without its memory traffic (see kernels_gemm_tiled.hip).
hipError_t launch_mfma_rate(uint64_t *dev_out, uint32_t slabs, bool lds, hipStream_t stream, uint64_t *flop);
hipError_t launch_grouped_f32(const Problem *p, uint32_t n, hipStream_t stream, uint64_t *launches);

// ---- depth-fused forward ------------------------------------------------------
// One launch for all layer depths of a round; a tile of depth l waits on a
// completion counter until its job's depth l-1 is stored.
constexpr uint32_t kChainMaxLayers = 6;       // layer depths one fused launch can hold
constexpr uint32_t kChainMaxProblems = 256;   // (job, layer) pairs of a launch, plus one filler per depth
constexpr uint32_t kChainJobSlots = 64;       // jobs per launch; their descriptors stay cached on the device
constexpr uint32_t kChainSpinLimit = 1u << 21;  // polls (about a microsecond each) before a wait gives up
struct ChainJob {
    int64_t key;                      // identifies the job across calls (descriptor cache)
    uint32_t M;                       // rows in this round, 1 .. 65535
    uint32_t n_layers;                // 1 .. kChainMaxLayers
    Problem layer[kChainMaxLayers];   // as for the per-depth launch (M is ignored)
};
struct Chain;                         // device table, counters, host mirror: one per pool
hipError_t chain_create(Chain **out);   // allocates about 20 KB of device memory
void chain_destroy(Chain *c);
// All launches of one Chain must be ordered on the device (one stream, or events):
// consecutive launches alternate between two sets of counters.
hipError_t launch_chain(Chain *c, const ChainJob *jobs, uint32_t n, bool bf16, uint32_t spin_limit,
                        hipStream_t stream, uint64_t *launches);
// 1 if a wait gave up in a launch that has completed since the last call (the
// caller has synchronized); clears the flag.
uint32_t chain_take_timeouts(Chain *c);

// ---- training step ------------------------------------------------------------
struct LossProblem {
    const float *logits;     // M x N
    const int32_t *labels;   // M
    void *grad;              // M x N bf16: (softmax - onehot) / M
    float *loss;             // mean cross-entropy
    float *row_loss;         // scratch, M floats
    uint32_t M, N;
};
struct UpdateProblem {
    const void *H;           // M x K bf16 (layer input)
    const void *G;           // M x N bf16 (gradient of the layer output)
    float *Wm;               // K x N float master weights, updated in place
    void *Wb;                // K x N bf16 working copy, rewritten
    uint32_t M, K, N;
    float lr;
};
hipError_t launch_softmax_xent(const LossProblem *p, uint32_t n, hipStream_t stream, uint64_t *launches);
// Wm <- Wm - lr * (H^T . G), Wb <- bf16(Wm), all problems in one launch.
hipError_t launch_grouped_dw_sgd(const UpdateProblem *p, uint32_t n, hipStream_t stream,
                                 uint64_t *launches);

}  // namespace salus
