// Shared declarations between the host-side C boundary (qadam_api.cpp) and the gfx950 kernels
// (qadam_kernels.hip).  Not part of the public interface.
#pragma once

#include <hip/hip_runtime_api.h>
#include <stdint.h>

#include "../../include/qadam.h"

namespace qadam {

// One unit of work of every kernel: a run of at most `tile_elems` consecutive elements that lies
// inside one layer segment.  Tiles start at a multiple of the tile size from the segment start, so
// the first element of a tile is the first element of a 32-element code group.
struct Tile {
    int64_t start;      // global flat index of the first element
    int64_t code_word;  // index of the tile's first uint32 in a worker's packed code buffer
    int32_t len;        // elements in the tile (1 .. tile_elems)
    int32_t seg;        // layer segment the tile belongs to
    int32_t flags;      // bit 0: start is not a multiple of 4 (no 128-bit accesses);
                        // bit 1: sampled tile of the filtered scale pass;
                        // bit 2: first tile of a small layer (see below); bit 3: a later tile of one;
                        // bits 8..9: zero words to append after the tile's codes (segment padding)
    int32_t layer_len;  // first tile of a small layer: elements of the whole layer; else 0
};
static_assert(sizeof(Tile) == 32, "tile records are read as two 128-bit scalar loads");

constexpr int kTileUnaligned = 1;
constexpr int kTileSampled = 2;
// A small layer (at most kSmallLayerElems elements) is handled by ONE workgroup in the kernels of the
// server-moments path: the workgroup of the layer's first tile takes the layer's scales itself (one read
// of g and e, which stay in cache) and then quantizes all of the layer's tiles, so these layers make a
// single trip through HBM and need no scale pass; the workgroups of the layer's other tiles exit at once.
// The worker-moments path (whose first pass produces the tile maxima anyway) ignores the two flags.
constexpr int kTileSmallHead = 4;
constexpr int kTileSmallBody = 8;
constexpr int kSmallLayerElems = 4 * 4096;
// A layer of at most kMediumLayerTiles tiles (small layers included) needs no launch of the kernel that
// folds tile maxima into scales: every workgroup that quantizes one of its tiles folds the layer's few
// tile maxima itself (they sit in L2), and the workgroup of the layer's first tile writes the scale out.
constexpr int kTileMedium = 16;
constexpr int kMediumLayerTiles = 640;
constexpr int kSampleStride = 64;   // every 64th tile of a layer (from its first) is a sampled tile
constexpr int kBlockThreads = 256;
constexpr int kDefaultTileElems = 4096;   // elements per tile (16 per lane of a 256-thread workgroup)

// Scalars of one launch, identical for every kernel.
struct StepScalars {
    int32_t  num_workers;
    int32_t  k_g, mu_bits, code_bits;   // Q_g: levels, bits of the level index, bits per code
    int32_t  k_x, wcode_bytes;          // Q_x
    int32_t  rounding, weight_ef, adam_flavor;
    uint32_t key0, key1;                // Philox key (seed)
    uint32_t step;                      // low 32 bits of t
    float    lr, beta1, beta2, eps;
    float    omb1, omb2;                // 1-beta, 1-theta_t (fp32 subtraction done on the host)
    float    lr1, sbc2;                 // flavour 1: lr / (1-beta^t), sqrt(1-theta^t)
    float    n_workers_f;               // (float)N
    float    inv_n;                     // 1/N, used when N is a power of two (then exact)
    int32_t  n_is_pow2;
};

// Pointer tables travel as kernel arguments.
struct WorkerPtrs {
    const float* grad[QADAM_MAX_WORKERS];
    float*       err[QADAM_MAX_WORKERS];
    uint32_t*    codes[QADAM_MAX_WORKERS];
    float*       scales[QADAM_MAX_WORKERS];
    float*       mw[QADAM_MAX_WORKERS];     // variant W only
    float*       vw[QADAM_MAX_WORKERS];
};

struct ServerPtrs {
    float* x;
    float* m;
    float* v;
    float* werr;        // may be null when weight_ef == 0
    void*  wcodes;
};

struct Launch {
    const Tile* tiles;      // device
    float*      inv_scales; // device, [num_workers][num_segments]: 1/s where the fast quotient is safe, else 0
    uint32_t*   tile_max;   // device, [num_workers][num_tiles]: per-tile max |p| as a bit pattern
    const int32_t* seg_tile_begin;  // device, [num_segments + 1]: first tile of every segment
    int32_t     num_tiles;
    int32_t     num_segments;
    int64_t     num_params;
    double*     tile_sum;   // device, [num_tiles]: per-tile partial sums of the norm diagnostic
    float*      err_bound;  // device, [num_workers][num_segments]: bound on |e| left by the last step
    uint32_t*   thr;        // device, [num_workers][num_segments]: thresholds of the filtered scale pass
    const int32_t* sample_tiles;    // device: indices of the sampled tiles
    int32_t     num_sample_tiles;
    uint32_t*   status;     // device status word
    bool        need_amax;   // server-moments path: some layer is neither small nor empty (else no tile-maxima launch)
    bool        need_reduce; // some layer has more than kMediumLayerTiles tiles, or is empty (else no scale-folding launch)
    hipStream_t stream;
};

// Launchers (defined in qadam_kernels.hip).  `first_worker`/`num` select the workers a launch covers.
// scales in two stages without atomics: per-tile maxima, then one workgroup per (worker, layer)
// reduces its tiles and also writes the reciprocal used by the fast quotient
hipError_t launch_amax(const Launch& L, const StepScalars& S, const WorkerPtrs& W, int first_worker, int num);
hipError_t launch_reduce_scales(const Launch& L, const StepScalars& S, const WorkerPtrs& W, int first_worker, int num);
hipError_t launch_amax_filtered(const Launch& L, const StepScalars& S, const WorkerPtrs& W, int first_worker, int num);
hipError_t launch_check_error_bounds(const Launch& L, const WorkerPtrs& W, int first_worker, int num);
hipError_t launch_worker_quantize(const Launch& L, const StepScalars& S, const WorkerPtrs& W, int worker);
hipError_t launch_server_step(const Launch& L, const StepScalars& S, const WorkerPtrs& W, const ServerPtrs& sp);
hipError_t launch_weight_quantize(const Launch& L, const StepScalars& S, const float* x, float* werr, void* wcodes);
hipError_t launch_weight_dequantize(const Launch& L, const StepScalars& S, const void* wcodes, void* xhat, bool half);
hipError_t launch_fused(const Launch& L, const StepScalars& S, const WorkerPtrs& W, const ServerPtrs& sp);
// Q_g = identity: the messages are fp32 values (variant S: the gradients; variant W: the parked
// update + error, whose buffers are then cleared)
hipError_t launch_plain_messages(const Launch& L, const StepScalars& S, const WorkerPtrs& W, const ServerPtrs& sp,
                                 bool variant_w);
hipError_t launch_layer_sumsq(const Launch& L, const float* a, const float* b, double* out);
// variant W
hipError_t launch_worker_moments_w(const Launch& L, const StepScalars& S, const WorkerPtrs& W, int first_worker, int num);
hipError_t launch_fused_w(const Launch& L, const StepScalars& S, const WorkerPtrs& W, const ServerPtrs& sp);
hipError_t launch_server_apply_w(const Launch& L, const StepScalars& S, const WorkerPtrs& W, float* x);


// Handle-free quantization of one segment (qadam_quantize_segment_noalloc): the per-tile maxima, the
// reciprocal scale and a status word live in a static device array, so nothing is allocated.
// noalloc_prepare looks up that array's address on the current device (once per device).
constexpr int64_t kNoallocMaxElems = QADAM_NOALLOC_MAX_ELEMS;
hipError_t noalloc_prepare();
hipError_t noalloc_quantize_segment(const StepScalars& S, int64_t n, const float* grad, float* err, uint32_t* codes,
                                    float* scale_out, hipStream_t stream);

}  // namespace qadam
