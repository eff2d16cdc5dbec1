// Internal declarations shared by the translation units of libsamo (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "samo.h"

namespace samo {

#ifndef SAMO_TILE_THREADS
#define SAMO_TILE_THREADS 256
#endif
#ifndef SAMO_TILE
#define SAMO_TILE 4096
#endif
#ifndef SAMO_U
#define SAMO_U 4
#endif
#ifndef SAMO_GLDS
#define SAMO_GLDS 0
#endif
#ifndef SAMO_ADAM_DWORD
#define SAMO_ADAM_DWORD 0
#endif
#ifndef SAMO_NT
#define SAMO_NT 9
#endif

constexpr int kThreads = 256;           // 4 wavefronts of 64 lanes per workgroup (flat and index kernels)
constexpr int kTileThreads = SAMO_TILE_THREADS;   // workgroup size of the tile kernels
constexpr int kSeg = SAMO_SEG_ELEMS;    // dense elements per seg_ptr entry
constexpr int kTile = SAMO_TILE;        // dense elements owned by one workgroup
constexpr int kSegsPerTile = kTile / kSeg;
#ifndef SAMO_CHUNK
#define SAMO_CHUNK 256
#endif
#ifndef SAMO_FLAT_THREADS
#define SAMO_FLAT_THREADS 64
#endif
constexpr int kChunk = SAMO_CHUNK;      // compressed elements per workgroup in the flat kernels
constexpr int kFlatThreads = SAMO_FLAT_THREADS;

static_assert(kTile % kSeg == 0, "a tile is a whole number of segments");
static_assert(kTile % (8 * kTileThreads) == 0, "a tile is written out as whole 16-byte vectors per thread");
static_assert(kChunk % (4 * kFlatThreads) == 0, "a chunk is whole float4 vectors per thread");

// Adam constants prepared on the host in double precision, rounded once to fp32.
struct AdamK {
    float lr, b1, b2, omb1, omb2, eps, wd;
    float rbc1, rbc2;   // 1 / (1 - beta^t)
    int l2, decoupled;
};

// Workgroup -> (layer, local tile or chunk) record of the batched launches.
struct WgRec {
    int32_t layer;
    int32_t local;
};

// Up to kIndexBatchJobs index-build jobs, passed to the kernels by value (kernel argument segment).
constexpr int kIndexBatchJobs = 48;
struct IndexBatch {
    int num;
    int wg_start[kIndexBatchJobs + 1];   // exclusive prefix of workgroups per job
    const uint8_t *mask[kIndexBatchJobs];
    int64_t n[kIndexBatchJobs];
    int32_t *idx[kIndexBatchJobs];
    int64_t cap[kIndexBatchJobs];
    int32_t *seg_ptr[kIndexBatchJobs];
    int64_t *nnz[kIndexBatchJobs];
};
static_assert(sizeof(IndexBatch) <= 3072, "the job table must fit the kernel argument segment");

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---- launchers (each returns hipGetLastError() after enqueueing) -----------------------
hipError_t launch_index_batch(const IndexBatch &batch, bool fill, hipStream_t s);
int64_t index_job_workgroups(int64_t n);
hipError_t launch_seg_ptr_from_idx(const int32_t *idx, int64_t nnz, int64_t n, int32_t *seg_ptr,
                                   hipStream_t s);
hipError_t launch_validate(const int32_t *idx, int64_t nnz, int64_t n, const int32_t *seg_ptr,
                           int32_t *ok, hipStream_t s);

hipError_t launch_decompress(const samo_layer &layer, hipStream_t s);
hipError_t launch_fused(const samo_layer &layer, float inv_scale, const AdamK &k, hipStream_t s);
hipError_t launch_gather(const samo_layer &layer, float inv_scale, hipStream_t s);
hipError_t launch_adam(const samo_layer &layer, const AdamK &k, hipStream_t s);

hipError_t launch_decompress_batched(const samo_layer *d_layers, const WgRec *d_tiles, int64_t ntiles,
                                     hipStream_t s);
hipError_t launch_fused_batched(const samo_layer *d_layers, const WgRec *d_tiles, int64_t ntiles,
                                float inv_scale, const AdamK &k, hipStream_t s);
hipError_t launch_gather_batched(const samo_layer *d_layers, const WgRec *d_chunks, int64_t nchunks,
                                 float inv_scale, hipStream_t s);
hipError_t launch_adam_batched(const samo_layer *d_layers, const WgRec *d_chunks, int64_t nchunks,
                               const AdamK &k, hipStream_t s);

hipError_t launch_copy(void *dst, const void *src, int64_t bytes, hipStream_t s);

}  // namespace samo
