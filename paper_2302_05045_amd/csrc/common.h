// Internal declarations shared by the translation units of libsamo (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "samo.h"

namespace samo {

// Launch shapes, chosen by measurement on MI355X.  A tile workgroup (256 threads) owns a run of
// whole segments of a layer of about equal weight kTileCost, where a segment weighs kSegCost plus
// kNnzCost per kept element: at 90 % pruning that is about 4 segments (4096 dense elements, 16
// per thread — 8 or 32 per thread lose 10-15 %), 3 at 80 %, 2 at 50 %, 5-6 where nothing is kept,
// one segment per workgroup in an unpruned layer; a model that keeps under 7 % is cut with
// twice the weight (kTileCostSparse), 8-9 segments at 95 % pruning.  The weights follow the fused step's traffic
// (4 bytes per dense element, 28 per kept one) with the dense side weighted up: swept over
// (4096..16384, 8..28, 20K..64K) on the GPT shapes, this choice is within 1 % of the best at 80, 90
// and 95 % uniform pruning and 6 % ahead of fixed 4096-element tiles on row-clustered masks.  Even
// weights per workgroup keep the traffic in flight per compute unit steady whatever the local
// density (clustered masks, mixed pruned and dense layers), so one occupancy target fits all.
// Flat kernels: one 64-lane wave per workgroup with one float4 per array.
constexpr int kThreads = 256;           // index kernels: 4 wavefronts per workgroup
constexpr int kTileThreads = 256;       // tile kernels that run an optimizer step
constexpr int kExpandThreads = 128;     // expansion only: little read traffic per tile, so more, smaller workgroups
                                        // per compute unit (+15 % over 256 threads; the step kernels lose with 128)
constexpr int kSeg = SAMO_SEG_ELEMS;    // dense elements per seg_ptr entry
constexpr int64_t kTileCost = 32768;    // target weight of one tile workgroup
constexpr int64_t kTileCostSparse = 65536;   // the same for a model with less than kSparseKeep of its elements kept: the
                                        // kernels that do not read the dense gradient move too few bytes per tile there
                                        // for the workgroups a compute unit holds (measured at 95 % pruning, weights
                                        // 32K / 48K / 64K: the compressed-gradient step 0.705 / 0.754 / 0.765 of peak,
                                        // the expansion 0.716 / 0.747 / 0.765, the fused step 0.81 throughout)
constexpr int64_t kTileCostSparse32 = 49152; // ... where the dense side is fp32 (single-precision SAMO): 0.78 / 0.80 / 0.73
constexpr double kSparseKeep = 0.07;
constexpr int64_t kSegCost = 6144;      // weight of a segment's dense side (fp16 gradient lines read, fp16 weights written)
constexpr int64_t kNnzCost = 24;        // weight of a kept element (idx, p, m, v read; p, m, v written)
constexpr int64_t kTileCostMax = 98304;   // what SAMO_KNOB_TILE_COST may ask for
constexpr int kMaxTileSegs = (int)((kTileCostMax + kSegCost - 1) / kSegCost);   // of any tile: reached where nothing is kept
// The tile weight of a model (a plan, or a layer launched by itself) and the segments its heaviest
// tile can hold: the size of the workgroups' LDS image, which is requested at launch.
int knob(int which, int fallback);
inline int64_t tile_cost_for(int64_t n, int64_t nnz, bool dense_fp32)
{
    const int64_t forced = (int64_t)knob(SAMO_KNOB_TILE_COST, 0) * 1024;      // tuning aid
    if (forced >= kSegCost && forced <= kTileCostMax) return forced;
    if (n > 0 && (double)nnz < kSparseKeep * (double)n) return dense_fp32 ? kTileCostSparse32 : kTileCostSparse;
    return kTileCost;
}
inline int tile_cost_segs(int64_t cost) { return (int)((cost + kSegCost - 1) / kSegCost); }
constexpr int kFlatThreads = 64;        // flat kernels over the compressed arrays
constexpr int kChunk = 256;             // compressed elements per workgroup in the flat kernels
constexpr int kStatReduceGrid = 1024;    // workgroups of the first level of the gradient-statistics reduction
constexpr int kTileUnrollFp32 = 4;      // compressed elements in flight per thread in the single-precision tile kernel

static_assert(kMaxTileSegs >= 1 && kMaxTileSegs < 256, "the segment count of a tile record is an 8-bit field");
static_assert(kSeg % 8 == 0, "a tile is written out as whole 16-byte vectors");
static_assert(kChunk % (4 * kFlatThreads) == 0, "a chunk is whole float4 vectors per thread");

// Optimizer constants prepared on the host in double precision, rounded once to fp32.
struct AdamK {
    float lr, b1, b2, omb1, omb2, eps, wd;
    float rbc1, rbc2;   // 1 / (1 - beta^t)
    int l2, decoupled;
};
struct OptK {
    AdamK adam;
    float sgd_lr, sgd_mu, sgd_wd;
};

// Clipping / overflow guard evaluated on the device from the gradient statistics.
struct GuardK {
    const samo_grad_stats *stats;   // NULL: no guard
    float max_norm;                 // <= 0: no clipping
    int skip;                       // leave all state untouched if stats->nonfinite
};

enum { kModeDecompress = 0, kModeStep = 1 };
enum { kGradDense = 0, kGradC16 = 1, kGradC32 = 2, kGradDense32 = 3 };   // where a step / the statistics read the gradient
enum { kOptAdam = 0, kOptSgd = 1 };
enum { kOutF32 = 0, kOutF16 = 1, kOutNone = 2 };        // what the flat gather kernel writes

// Workgroup -> work record of the batched launches.  Chunk records (flat kernels): local = chunk
// index within the layer.  Tile records: local = first segment | number of segments << 24 (a
// layer has at most 2^21 segments).
struct WgRec {
    int32_t layer;
    uint32_t local;
};
constexpr int kRecSegShift = 24;

// One (sum of squares, non-finite flag) partial per workgroup of a flat launch.
struct StatPartial {
    double sum_squares;
    int64_t nonfinite;
};

// Process-wide tuning and testing knobs (samo_debug_set); `dflt` where a knob holds SAMO_KNOB_DEFAULT.
int knob(int which, int dflt);

// Up to kIndexBatchJobs index-build jobs, passed to the kernels by value (kernel argument segment).
constexpr int kIndexBatchJobs = 48;
constexpr int kIndexSpinLimit = 1 << 20;   // about a second of polling
struct IndexBatch {
    int num;
    int wg_start[kIndexBatchJobs + 1];   // exclusive prefix of workgroups per job
    const uint8_t *mask[kIndexBatchJobs];
    int64_t n[kIndexBatchJobs];
    int32_t *idx[kIndexBatchJobs];
    int64_t cap[kIndexBatchJobs];
    int32_t *seg_ptr[kIndexBatchJobs];
    int64_t *nnz[kIndexBatchJobs];
    int passes;                          // 64 KiB passes a workgroup makes over its block: 1, 2 or 4
    int spin_limit;                      // polls of a missing predecessor before a workgroup gives up
    int64_t *ticket;                     // the nnz of the job that owns the last workgroup: zero before the
                                         // launch, counts the workgroups as they start, final once that one ends
};
static_assert(sizeof(IndexBatch) <= 3072, "the job table must fit the kernel argument segment");

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---- launchers (each returns hipGetLastError() after enqueueing) -----------------------
hipError_t launch_index_batch(const IndexBatch &batch, bool fill, hipStream_t s);
int64_t index_job_workgroups(int64_t n, int passes);
int index_passes_for(int64_t mask_bytes, int compute_units);
hipError_t launch_seg_ptr_from_idx(const int32_t *idx, int64_t nnz, int64_t n, int32_t *seg_ptr,
                                   hipStream_t s);
hipError_t launch_validate(const int32_t *idx, int64_t nnz, int64_t n, const int32_t *seg_ptr,
                           int32_t *ok, hipStream_t s);

// `layers`/`recs` NULL: single-layer launch of `one`; else batched over the plan's tables.
struct LaunchSet {
    samo_layer one;
    const samo_layer *layers;
    const WgRec *recs;
    int64_t wgs;
    int segs_per_tile;   // single-layer tile launches: workgroup b owns segments [b * this, (b + 1) * this)
    float keep;          // kept fraction nnz / n of the work (plan average); steers the flat kernels' occupancy target
    int max_segs;        // tile launches: segments the workgroups' LDS image holds (no tile of the launch has more)
};
// Segments per tile of a single-layer launch, from the layer's average density.
int single_layer_tile_segs(int64_t n, int64_t nnz, bool dense, bool dense_fp32);
// Up to kPlanBatchLayers layer descriptors of a plan with the starts of their tile and chunk records,
// passed to plan_write_kernel by value: the host table reaches the device without a copy.
constexpr int kPlanBatchLayers = 24;
struct PlanBatch {
    int first, count;                                 // layers [first, first + count) of the plan
    samo_layer layer[kPlanBatchLayers];
    int64_t tile_start[kPlanBatchLayers + 1];         // entry `count` is the start of layer first + count
    int64_t chunk_start[kPlanBatchLayers + 1];
};
static_assert(sizeof(PlanBatch) <= 3072, "the layer table must fit the kernel argument segment");
// Device tables of a plan inside the caller's workspace.
struct PlanTables {
    samo_layer *layers;
    int64_t *tile_start, *chunk_start;                // num_layers + 1 entries each
    WgRec *tiles, *chunks;
};
hipError_t launch_plan_write(const PlanBatch &batch, const PlanTables &t, hipStream_t s);
// Fills the tile and chunk records of every layer (reads the tables plan_write_kernel wrote and the layers' seg_ptr).
hipError_t launch_plan_records(const PlanTables &t, int num_layers, int64_t ntiles, int64_t nchunks, int64_t tile_cost,
                               hipStream_t s);
hipError_t launch_tile(int mode, int gsrc, int opt, const LaunchSet &ls, float inv_scale, const OptK &k,
                       const GuardK &guard, hipStream_t s);
hipError_t launch_tile_fp32(const LaunchSet &ls, float factor, const OptK &k, const GuardK &guard, hipStream_t s);
hipError_t launch_gather(int out, int src, const LaunchSet &ls, float inv_scale, int accumulate,
                         StatPartial *partials, hipStream_t s);
hipError_t launch_flat_step(int opt, const LaunchSet &ls, const OptK &k, const GuardK &guard, hipStream_t s);
int64_t stats_workspace_partials(int64_t gather_wgs);
hipError_t launch_stats_finalize(StatPartial *partials, int64_t gather_wgs, samo_grad_stats *out, hipStream_t s);

// Weight gradients dY^T X of up to kWgradMaxJobs linear layers, each gathered at its layer's index, in
// one launch (out_kind: kOutF32 or kOutF16; gc of that type).
constexpr int kWgradMaxJobs = SAMO_WGRAD_MAX_JOBS;
struct WgradJob {
    const _Float16 *dy;      // tokens x out
    const _Float16 *x;       // tokens x in
    int64_t tokens;
    int out, in;
    const int32_t *idx;
    const int32_t *seg_ptr;
    int64_t nnz;
    void *gc;
};
hipError_t launch_wgrad(int out_kind, const WgradJob *jobs, int count, float inv_scale, int accumulate, hipStream_t s);
// Function attributes of the weight-gradient kernels and the compute-unit count of the current device (once per device).
hipError_t wgrad_configure(int *cus);
constexpr int kMfmaRateWaves = 8;          // waves per workgroup of launch_mfma_rate, 8 MFMAs of 32 x 32 x 16 each per iteration
hipError_t launch_mfma_rate(int64_t iters, float *sink, int workgroups, hipStream_t s);

hipError_t launch_copy(void *dst, const void *src, int64_t bytes, hipStream_t s);

}  // namespace samo
