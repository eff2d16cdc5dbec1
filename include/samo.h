/*
 * samo.h — C ABI of libsamo: the per-iteration compressed-parameter pipeline of
 * Sparsity-aware Memory Optimization (SAMO; Singh & Bhatele, "Exploiting
 * Sparsity in Pruned Neural Networks to Optimize Large Model Training",
 * Section III) for one AMD MI355X (gfx950).
 *
 * Storage (Section III-A, III-B).  For every pruned layer, with N = number of
 * elements of its flattened 1-D view and nnz = number of unpruned elements:
 *   idx      int32[nnz]   ascending flat positions of the unpruned elements
 *                         (the paper's ind_i), shared by all compressed tensors
 *   p, m, v  float[nnz]   fp32 master parameters and the two Adam states, values
 *                         at the unpruned positions only (theta32, os)
 *   gc       float[nnz]   compressed, up-cast, unscaled gradient (grad theta32)
 *   gc16     fp16[nnz]    compressed half-precision gradient (grad theta16), still
 *                         multiplied by the loss scale; the data-parallel
 *                         all-reduce message of Section IV-A
 *   w        fp16[N]      dense half-precision parameters (theta16) with +0
 *                         stored explicitly at every pruned position
 *   g        fp16[N]      dense half-precision gradient as backward produced it
 *   w32, g32 float[N]     single-precision SAMO only: dense fp32 parameters (zeros stored
 *                         explicitly) and dense fp32 gradient
 *   seg_ptr  int32[ceil(N / SAMO_SEG_ELEMS) + 1]
 *                         seg_ptr[s] = #{ i : idx[i] < s * SAMO_SEG_ELEMS };
 *                         seg_ptr[last] = nnz.  Not in the paper: a small table
 *                         (4 bytes per 1024 dense elements) that lets a
 *                         workgroup owning a dense tile find its slice of the
 *                         compressed arrays without searching.
 * fp16 values cross this boundary as uint16_t bit patterns (IEEE binary16).
 *
 * Conventions common to every entry point
 *   - Pointers named d_* are DEVICE pointers, h_* are HOST pointers.  The caller
 *     owns every buffer, workspaces included.  The library is stateless: it
 *     allocates nothing, frees nothing and copies nothing between host and
 *     device; host tables (layer descriptors, job lists) reach the device inside
 *     kernel arguments.
 *   - `stream` is a hipStream_t passed as void*; NULL is the default stream.
 *     Every call only enqueues kernels on `stream` and returns; nothing
 *     synchronises, nothing runs on another stream, so every entry point that
 *     takes a stream can be captured into a HIP graph (after one samo_init).
 *     Outputs (including *d_nnz) are valid once the stream reaches that point.
 *   - No exceptions cross this boundary, nothing is printed, errno is untouched and
 *     no environment variable is read.
 *   - Arguments are validated on the host BEFORE anything is enqueued.  On a
 *     negative status nothing was launched and no output was touched.
 *   - Sizes: 0 <= N <= 2^31 - 1 per layer (the index is 32-bit, Section III-B);
 *     0 <= nnz <= N.  N = 0 and nnz = 0 are valid and do nothing / zero-fill;
 *     pointers to arrays of nnz elements may be NULL when nnz == 0.
 *   - Alignment: every array pointer must be 16-byte aligned (SAMO_ERR_ALIGN).
 *   - Preconditions NOT checked on the hot path (results undefined if violated;
 *     samo_validate_index checks them): idx strictly ascending, 0 <= idx[i] < N,
 *     seg_ptr consistent with idx.  Strictly ascending indices make scatter
 *     race-free without atomics.
 *   - Aliasing: w and g of a layer must not overlap; p, m, v are updated in place.
 *   - Every result is deterministic: same inputs give the same bits.
 */
#ifndef SAMO_H
#define SAMO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SAMO_ABI_VERSION 4
#define SAMO_SEG_ELEMS 1024 /* dense elements per seg_ptr entry */

typedef int32_t samo_status;
enum {
    SAMO_OK = 0,
    SAMO_ERR_NULL = -1,  /* a required pointer is NULL */
    SAMO_ERR_SIZE = -2,  /* N or nnz out of range, or capacity/length too small */
    SAMO_ERR_ARG = -3,   /* invalid hyper-parameter or scale */
    SAMO_ERR_WORKSPACE = -4, /* workspace NULL or smaller than the *_workspace_bytes call reports */
    SAMO_ERR_ALIGN = -5, /* pointer not 16-byte aligned */
    SAMO_ERR_INDEX = -6, /* never returned by a call (the index is checked on the device only): the
                            value a caller reports when *d_nnz reads -1 after an index build, or
                            *d_ok reads 0 after samo_validate_index */
    SAMO_ERR_HIP = -7,   /* HIP runtime reported an error on launch */
    SAMO_ERR_PLAN = -8   /* plan lacks a buffer this entry point needs */
};

/* Static string for a status code (never NULL). */
const char *samo_status_string(samo_status s);
int32_t samo_abi_version(void);
/* Optional set-up for the CURRENT device, outside stream capture: sets the HIP function
 * attributes the weight-gradient kernels need and resolves the device address of the library's
 * static scratch array.  Entry points do the same on their first call on a device, which must then
 * not be a captured one; after samo_init every call is pure kernel launches.  Idempotent. */
samo_status samo_init(void);
/* ceil(n / SAMO_SEG_ELEMS) + 1, the required length of seg_ptr; -1 if n is out of range. */
int64_t samo_seg_ptr_len(int64_t n);

/* Adam hyper-parameters (Kingma & Ba; the optimizer assumed by Section III-D).
 * step >= 1 is Adam's t; eps > 0 is added after the square root of the
 * bias-corrected second moment; 0 <= beta < 1.  weight_decay is added to the
 * gradient (decoupled_wd = 0, L2) or applied to the parameter directly
 * (decoupled_wd = 1, AdamW as used for the paper's GPT runs, Section V). */
typedef struct {
    float lr, beta1, beta2, eps, weight_decay;
    int32_t decoupled_wd;
    int32_t step;
} samo_adam_cfg;

/* SGD with momentum (one fp32 state per parameter, held in `m`; the paper's CNN runs use SGD,
 * Section V, and Section III-D notes that SAMO extends to other optimizers):
 * buf = momentum * buf + g (+ weight_decay * p); p = p - lr * buf; buf starts at zero. */
typedef struct {
    float lr, momentum, weight_decay;
} samo_sgd_cfg;

/* Gradient statistics of a whole model, DEVICE resident: the sum of squares of the unscaled
 * compressed gradient (for clipping by global norm; the paper trains with gradient clipping,
 * Section V) and whether any value is NaN or infinite (the overflow check of mixed-precision
 * training).  Written by the entry points that take a d_stats argument. */
typedef struct {
    double sum_squares;
    int32_t nonfinite;
    int32_t reserved;
} samo_grad_stats;

/* Optional guard of a batched optimizer step, evaluated on the device (no host round trip):
 * every gradient is multiplied by min(1, max_grad_norm / (sqrt(sum_squares) + 1e-6)) when
 * max_grad_norm > 0, and when skip_on_nonfinite != 0 and the statistics report a non-finite
 * value the step does nothing at all (p, m, v and w keep their contents).  d_stats must have
 * been written earlier on the same stream.  A NULL guard means no clipping and no skipping. */
typedef struct {
    const samo_grad_stats *d_stats;
    float max_grad_norm;
    int32_t skip_on_nonfinite;
} samo_step_guard;

/* ---------------------------------------------------------------- index (ind_i, Section III / III-B)
 * The pruning algorithm's output is taken as a byte mask over the flattened
 * layer: mask[j] != 0 means element j is unpruned.
 *
 * The construction needs one device workspace per layer, and that workspace is
 * seg_ptr itself: samo_index_workspace_bytes reports 4 * samo_seg_ptr_len(n).
 * Unlike an ordinary workspace its contents are an output (the table above) that
 * the expansion and step entries read later, so the entries name it d_seg_ptr
 * and give it its element type.
 *
 * samo_count_nonzero: fills d_seg_ptr[0 .. samo_seg_ptr_len(n)) and *d_nnz.
 * samo_build_index:   the same, and writes the ascending positions to d_idx.
 *   If nnz > idx_capacity only the first idx_capacity positions are stored;
 *   *d_nnz still holds the true count, so the caller can detect it.
 *   d_idx may be NULL only if idx_capacity == 0.
 * Typical use: count, read *d_nnz, allocate idx, build; or build with capacity n.
 * The mask is read once: workgroups pass the running count along a chain kept in
 * d_seg_ptr, waiting for their predecessors for a bounded time.  Should that wait
 * ever run out (it cannot unless the device stops scheduling running workgroups)
 * *d_nnz is set to -1 and d_seg_ptr / d_idx are incomplete.  While the call is in
 * flight d_seg_ptr and *d_nnz hold intermediate values; the outputs of different
 * jobs of one call must not overlap. */
samo_status samo_index_workspace_bytes(int64_t n, size_t *bytes);
samo_status samo_count_nonzero(const uint8_t *d_mask, int64_t n, int32_t *d_seg_ptr,
                               int64_t *d_nnz, void *stream);
samo_status samo_build_index(const uint8_t *d_mask, int64_t n, int32_t *d_idx,
                             int64_t idx_capacity, int32_t *d_seg_ptr, int64_t *d_nnz,
                             void *stream);
/* The same for many layers with a handful of launches (two per group of up to 48 jobs), so
 * that small layers do not pay their own launches.  h_jobs is a HOST array of jobs
 * holding DEVICE pointers; a job with idx == NULL and idx_capacity == 0 only counts.  Every job
 * is validated before anything is enqueued. */
typedef struct {
    const uint8_t *mask;
    int64_t n;
    int32_t *idx;
    int64_t idx_capacity;
    int32_t *seg_ptr;
    int64_t *nnz;
} samo_index_job;
samo_status samo_build_index_batched(const samo_index_job *h_jobs, int32_t num_jobs, void *stream);
/* seg_ptr for an index that came from elsewhere (e.g. straight from a pruner). */
samo_status samo_build_seg_ptr(const int32_t *d_idx, int64_t nnz, int64_t n,
                               int32_t *d_seg_ptr, void *stream);
/* *d_ok = 1 if idx is strictly ascending within [0, n) and (when d_seg_ptr is
 * not NULL) seg_ptr matches it; else 0. */
samo_status samo_validate_index(const int32_t *d_idx, int64_t nnz, int64_t n,
                                const int32_t *d_seg_ptr, int32_t *d_ok, void *stream);

/* ---------------------------------------------------------------- expansion (Section III-C, optimizer step)
 * w[idx[i]] = fp16(p[i]) (round to nearest even, subnormals kept, overflow to
 * infinity); every other element of w[0..n) = +0, whatever w held before. */
samo_status samo_decompress(const float *d_p, const int32_t *d_idx, const int32_t *d_seg_ptr,
                            int64_t nnz, uint16_t *d_w, int64_t n, void *stream);

/* ---------------------------------------------------------------- gradient compression (Section III-C, backward pass;
 * merged with the fp32 up-cast of the optimizer step and loss-scale division)
 * gc[i] = float(g[idx[i]]) * inv_loss_scale — one exact conversion, one fp32
 * multiply.  Gradient values at pruned positions are ignored.
 * inv_loss_scale must be finite and > 0. */
samo_status samo_gather_grads(const uint16_t *d_g, int64_t n, const int32_t *d_idx,
                              int64_t nnz, float inv_loss_scale, float *d_gc, void *stream);

/* The stored compressed half-precision gradient (Section III-A) — what a data-parallel
 * all-reduce would send (Section IV-A).  accumulate == 0: gc16[i] = g[idx[i]] (pure movement);
 * accumulate != 0: gc16[i] = fp16(gc16[i] + g[idx[i]]), one correctly rounded half addition
 * (a further micro-batch, Section II-E).  The loss scale stays in the values. */
samo_status samo_gather_grads_fp16(const uint16_t *d_g, int64_t n, const int32_t *d_idx,
                                   int64_t nnz, uint16_t *d_gc16, int32_t accumulate, void *stream);

/* ---------------------------------------------------------------- optimizer on compressed state (Section III-C, III-D)
 * One Adam step over p, m, v [0..nnz) with gradient gc, all fp32, in place. */
samo_status samo_adam_step(float *d_p, float *d_m, float *d_v, const float *d_gc, int64_t nnz,
                           const samo_adam_cfg *h_cfg, void *stream);
/* One SGD-momentum step over p, buf [0..nnz) with gradient gc. */
samo_status samo_sgd_step(float *d_p, float *d_buf, const float *d_gc, int64_t nnz,
                          const samo_sgd_cfg *h_cfg, void *stream);

/* ---------------------------------------------------------------- fused optimizer phase (Section III-C: compress + up-cast,
 * optimizer, 16-bit copy, expansion — in one pass)
 * Equivalent to samo_gather_grads -> samo_adam_step -> samo_decompress without
 * materialising gc or the temporary compressed fp16 copy.
 * Dense (unpruned) layer: d_idx == NULL, d_seg_ptr == NULL and nnz == n. */
samo_status samo_fused_step(const uint16_t *d_g, uint16_t *d_w, int64_t n, const int32_t *d_idx,
                            const int32_t *d_seg_ptr, int64_t nnz, float *d_p, float *d_m,
                            float *d_v, float inv_loss_scale, const samo_adam_cfg *h_cfg,
                            void *stream);

/* The optimizer phase as it runs AFTER a gradient all-reduce (Section IV-A, Section III-C):
 * up-cast of the compressed fp16 gradient with the loss-scale division, Adam on the compressed
 * state, 16-bit copy and expansion.  Equals samo_fused_step when gc16 holds g at idx. */
samo_status samo_adam_expand_step(const uint16_t *d_gc16, uint16_t *d_w, int64_t n, const int32_t *d_idx,
                                  const int32_t *d_seg_ptr, int64_t nnz, float *d_p, float *d_m,
                                  float *d_v, float inv_loss_scale, const samo_adam_cfg *h_cfg,
                                  void *stream);
/* samo_fused_step with SGD momentum instead of Adam (state in d_buf). */
samo_status samo_fused_sgd_step(const uint16_t *d_g, uint16_t *d_w, int64_t n, const int32_t *d_idx,
                                const int32_t *d_seg_ptr, int64_t nnz, float *d_p, float *d_buf,
                                float inv_loss_scale, const samo_sgd_cfg *h_cfg, void *stream);

/* ---------------------------------------------------------------- single-precision SAMO
 * Section III notes that the optimizations apply to single-precision training as well.  There
 * theta32 is the only copy of the parameters and stays dense with explicit zeros (w32, n floats:
 * what forward and backward use); the dense fp32 gradient g32 is read at the kept positions; the
 * optimizer state m, v is compressed; there are no 16-bit copies and no loss scale.  One optimizer
 * phase: for every kept position j = idx[i]:  g = g32[j] * grad_factor (one fp32 multiply; 1.0f
 * unless the gradient is to be scaled), one Adam step on (w32[j], m[i], v[i]).  Every other
 * element of w32[0..n) is +0 on exit, whatever it held.  grad_factor must be finite and > 0.
 * Dense (unpruned) layer: d_idx == NULL, d_seg_ptr == NULL and nnz == n. */
samo_status samo_fused_step_fp32(const float *d_g32, float *d_w32, int64_t n, const int32_t *d_idx,
                                 const int32_t *d_seg_ptr, int64_t nnz, float *d_m, float *d_v,
                                 float grad_factor, const samo_adam_cfg *h_cfg, void *stream);

/* ---------------------------------------------------------------- whole-model (batched) forms
 * One launch covers every layer, so small layers do not pay a launch and a
 * tail each.  A plan describes the model to those launches: the layer
 * descriptors and the workgroup-to-work maps, all of them in a device workspace
 * the CALLER provides.  The maps split every pruned layer into runs of segments
 * that move about equal numbers of bytes, which they read off seg_ptr.
 *
 * samo_plan_workspace_bytes: the workspace size for these layers (host
 *   arithmetic on n, nnz and on whether seg_ptr is NULL; nothing is dereferenced).
 *   It is an upper bound: samo_plan_init may need a little less (a model that
 *   keeps under 7 % of its elements is cut into heavier tiles when its dense
 *   side is fp16 than when it is fp32, and the size is that of the lighter ones).
 * samo_plan_init: validates h_layers (a HOST array of descriptors holding
 *   DEVICE pointers), then enqueues on `stream` the kernels that write the
 *   tables into d_workspace (the descriptors travel in kernel arguments, a few
 *   launches of up to 24 layers each) and fills *plan, a small host struct the
 *   caller owns.  Nothing is allocated, copied or synchronised; nothing has to be
 *   destroyed.  The kernels read every layer's seg_ptr in stream order, so an
 *   index build enqueued on the same stream just before is seen complete, and
 *   the whole sequence build index -> init plan -> step can sit in one HIP graph.
 *   *plan is usable by later calls on the same stream as soon as this returns
 *   (by calls on other streams once they wait for this one); it stays valid while
 *   the workspace and the layers' buffers are, until the index changes.
 * nnz of a descriptor is the CAPACITY of the layer's compressed arrays, and the
 *   launch sizes follow from it.  The number of kept elements the kernels use is
 *   what the layer's seg_ptr holds in its last entry when samo_plan_init's
 *   kernels run: the same number, unless the index was rebuilt with fewer kept
 *   elements (a captured graph replayed after re-pruning), which is valid.  An
 *   index with more kept elements than the capacity is cut off there.
 * A descriptor with idx == NULL (then seg_ptr == NULL and nnz == n) is a dense
 * layer.  Buffers an entry point does not use may be NULL in the descriptor
 * (e.g. gc for the fused step); an entry point that needs a missing one returns
 * SAMO_ERR_PLAN.  After re-pruning: rebuild the index, call samo_plan_init again
 * (the same workspace can be reused once earlier work on it has finished). */
typedef struct {
    int64_t n, nnz;
    const int32_t *idx;
    const int32_t *seg_ptr;
    float *p, *m, *v;
    uint16_t *w;
    const uint16_t *g;
    float *gc;
    uint16_t *gc16;
    float *w32;        /* single-precision SAMO: dense fp32 parameters (theta32 with explicit zeros) */
    const float *g32;  /* single-precision SAMO: dense fp32 gradient */
} samo_layer;

/* Filled by samo_plan_init; read-only for the caller.  Plain data: copy it freely, no call frees it. */
typedef struct {
    const void *d_layers;   /* device: samo_layer[num_layers], nnz as found in seg_ptr */
    const void *d_tiles;    /* device: one record per workgroup of the tile kernels */
    const void *d_chunks;   /* device: one record per workgroup of the flat kernels */
    int64_t num_tiles, num_chunks;
    int64_t n_total, nnz_total;   /* sums over the descriptors as given */
    int32_t num_layers;
    uint32_t buffers;       /* bits 0-8: which arrays every layer of the plan provides; bits 16-23: the most
                               segments one tile of the plan holds (sizes the tile kernels' LDS request) */
} samo_plan;

samo_status samo_plan_workspace_bytes(const samo_layer *h_layers, int32_t num_layers, size_t *bytes);
samo_status samo_plan_init(const samo_layer *h_layers, int32_t num_layers, void *d_workspace,
                           size_t workspace_bytes, void *stream, samo_plan *plan);

/* Gradient statistics need one (sum, flag) partial per workgroup: *bytes is the size of the
 * device workspace the entry points with a d_stats argument require for this plan
 * (SAMO_ERR_WORKSPACE if it is missing or smaller). */
samo_status samo_plan_stats_workspace_bytes(const samo_plan *plan, size_t *bytes);

samo_status samo_decompress_batched(const samo_plan *plan, void *stream);
/* Gather entries: when d_stats != NULL the statistics of what was gathered (for fp16: of the
 * values after accumulation), multiplied by inv_loss_scale, are reduced on the way — the pass
 * over the gradient is not repeated.  d_workspace/workspace_bytes as reported above; both are
 * ignored when d_stats == NULL.  The reduction order is fixed: results are deterministic. */
samo_status samo_gather_batched(const samo_plan *plan, float inv_loss_scale, samo_grad_stats *d_stats,
                                void *d_workspace, size_t workspace_bytes, void *stream);
samo_status samo_gather_fp16_batched(const samo_plan *plan, int32_t accumulate, float inv_loss_scale,
                                     samo_grad_stats *d_stats, void *d_workspace, size_t workspace_bytes,
                                     void *stream);
/* Statistics only, for callers that run the fully fused step: source selects what is read —
 * 0: the dense fp16 gradient g at idx, 1: gc16, 2: gc (fp32, already unscaled: pass 1.0f),
 * 3: the dense fp32 gradient g32 at idx (single-precision SAMO; the factor plays grad_factor). */
samo_status samo_grad_stats_batched(const samo_plan *plan, int32_t source, float inv_loss_scale,
                                    samo_grad_stats *d_stats, void *d_workspace, size_t workspace_bytes,
                                    void *stream);
/* samo_grad_stats_batched for callers that cannot allocate or hand over a workspace (code under
 * HIP graph capture, tight serving loops, harnesses that forbid allocation): the partials go to a
 * static array in the library's own device image (samo_static_scratch_bytes() = 16 MiB, held by
 * every GPU the library runs on until the process ends) instead of a caller workspace.  The call
 * allocates and frees nothing.  A plan whose samo_plan_stats_workspace_bytes exceeds that size
 * (more than about 268 M kept elements) is rejected with SAMO_ERR_SIZE before anything is enqueued.
 * Results are bit-equal to samo_grad_stats_batched.  All calls on one GPU share the one array:
 * calls that overlap in time on the same GPU (different streams) race and must be ordered by the
 * caller.  The array's device address is looked up on the first call on a device (or by
 * samo_init); make that call outside stream capture. */
size_t samo_static_scratch_bytes(void);
samo_status samo_grad_stats_batched_static(const samo_plan *plan, int32_t source, float inv_loss_scale,
                                           samo_grad_stats *d_stats, void *stream);
/* Optimizer entries; h_guard may be NULL. */
samo_status samo_adam_batched(const samo_plan *plan, const samo_adam_cfg *h_cfg,
                              const samo_step_guard *h_guard, void *stream);
samo_status samo_fused_step_batched(const samo_plan *plan, float inv_loss_scale,
                                    const samo_adam_cfg *h_cfg, const samo_step_guard *h_guard,
                                    void *stream);
samo_status samo_adam_expand_batched(const samo_plan *plan, float inv_loss_scale,
                                     const samo_adam_cfg *h_cfg, const samo_step_guard *h_guard,
                                     void *stream);
samo_status samo_fused_sgd_step_batched(const samo_plan *plan, float inv_loss_scale,
                                        const samo_sgd_cfg *h_cfg, const samo_step_guard *h_guard,
                                        void *stream);
/* samo_fused_step_fp32 over every layer of the plan (descriptors with w32, g32, m, v; p is not used
 * and may be NULL in a plan that serves only this entry). */
samo_status samo_fused_step_fp32_batched(const samo_plan *plan, float grad_factor,
                                         const samo_adam_cfg *h_cfg, const samo_step_guard *h_guard,
                                         void *stream);

/* ---------------------------------------------------------------- compression inside the backward pass
 * (Section III-C: a layer's dense gradient is compressed as soon as the backward
 * pass has produced it; Section VI-C, discussion of the compute overhead: fusing
 * that compression into the backward kernel is what would remove it.)
 * Weight gradient of a fully connected layer Y = X W^T with W of out x in
 * (Section I describes the layer as a linear transform of its input; the layout
 * convention is the frameworks' usual one), formed and compressed in one kernel: with
 *   dW[o][i] = sum over t < tokens of dY[t][o] * X[t][i]   (fp16 products, fp32 sums),
 * position o * in + i of the layer, and h = fp16(dW) rounded once to nearest
 * even (the value the dense fp16 gradient tensor would have held),
 *   samo_wgrad_gather:       gc[k]   = float(h[idx[k]]) * inv_loss_scale
 *   samo_wgrad_gather_fp16:  gc16[k] = h[idx[k]], or fp16(gc16[k] + h[idx[k]]) if accumulate != 0
 * i.e. samo_gather_grads / samo_gather_grads_fp16 applied to that tensor, which
 * is never written to memory.  The order of the fp32 summation over tokens is
 * the kernel's own: results agree with any other order within tokens * 2^-23 *
 * sum_t |dY[t][o] * X[t][i]| before the rounding to fp16.
 * d_dy: device, tokens x out row-major fp16; d_x: device, tokens x in row-major
 * fp16; both read only and 16-byte aligned.  out and in must be multiples of 8
 * with out * in < 2^31; tokens >= 0 (0: every dW is +0).  d_idx / d_seg_ptr
 * describe the layer of n = out * in elements as everywhere else; d_idx may be
 * NULL only when nnz == out * in (unpruned layer), d_seg_ptr is required
 * whenever d_idx is given.  Nothing is written when nnz == 0.
 * The first call on a device configures the kernels' LDS size (a HIP function
 * attribute): call samo_init, or make that first call, outside stream capture;
 * later calls only enqueue. */
samo_status samo_wgrad_gather(const uint16_t *d_dy, const uint16_t *d_x, int64_t tokens,
                              int64_t out, int64_t in, const int32_t *d_idx,
                              const int32_t *d_seg_ptr, int64_t nnz, float inv_loss_scale,
                              float *d_gc, void *stream);
samo_status samo_wgrad_gather_fp16(const uint16_t *d_dy, const uint16_t *d_x, int64_t tokens,
                                   int64_t out, int64_t in, const int32_t *d_idx,
                                   const int32_t *d_seg_ptr, int64_t nnz, uint16_t *d_gc16,
                                   int32_t accumulate, void *stream);

/* The same for several layers in one call: the tiles of all the jobs' layers are dealt to the
 * compute units as one list, so that a layer whose own tiles would end in a partly filled round
 * shares that round with the next layer (the four matrices of a GPT-3 2.7B transformer layer at
 * 2048 tokens: 0.35 ms in one call against 0.42 ms in four).  The caller holds dY and X of all
 * the jobs' layers until the call — it trades that memory for the time.  Each job is one layer
 * with the arguments of samo_wgrad_gather / samo_wgrad_gather_fp16 (d_gc: fp32 for
 * samo_wgrad_gather_batched, fp16 for samo_wgrad_gather_fp16_batched; tokens may differ between
 * jobs); h_jobs is a host array that is read before the call returns; count <=
 * SAMO_WGRAD_MAX_JOBS; jobs with nnz == 0 are skipped.  A call with one job is the unbatched
 * entry.  Any invalid job rejects the whole call before anything is launched. */
#define SAMO_WGRAD_MAX_JOBS 8
typedef struct samo_wgrad_job {
    const uint16_t *d_dy;         /* device, tokens x out fp16 */
    const uint16_t *d_x;          /* device, tokens x in fp16 */
    int64_t tokens, out, in;
    const int32_t *d_idx;         /* device, nnz; NULL for an unpruned layer */
    const int32_t *d_seg_ptr;     /* device; required with d_idx */
    int64_t nnz;
    void *d_gc;                   /* device, nnz elements of the entry's output type */
} samo_wgrad_job;
samo_status samo_wgrad_gather_batched(int32_t count, const samo_wgrad_job *h_jobs,
                                      float inv_loss_scale, void *stream);
samo_status samo_wgrad_gather_fp16_batched(int32_t count, const samo_wgrad_job *h_jobs,
                                           int32_t accumulate, void *stream);

/* ---------------------------------------------------------------- byte accounting (Section III-D, Eq. 1-5)  [host only]
 * paper_default = 20 * n_total; paper_samo = 24 * nnz_total + 2 * n_total;
 * resident = what this library's fused pipeline keeps allocated:
 * 16 * nnz_total (idx, p, m, v) + 2 * n_total (w) + 4 bytes per seg_ptr entry
 * is NOT included (layer-count dependent); any output pointer may be NULL. */
samo_status samo_memory_model(int64_t n_total, int64_t nnz_total, int64_t *paper_default,
                              int64_t *paper_samo, int64_t *resident);

/* ---------------------------------------------------------------- diagnostics
 * Plain device-to-device copy of `bytes` bytes (multiple of 16) with the same
 * launch shape as the pipeline's kernels: measures the achievable HBM stream
 * rate and calibrates hardware byte counters.  Not part of the method. */
samo_status samo_stream_copy(void *d_dst, const void *d_src, int64_t bytes, void *stream);
/* Issues `iters` rounds of eight independent 32x32x16 fp16 matrix instructions per wave from
 * registers, 8 waves per workgroup, `workgroups` workgroups (one per compute unit fills the
 * device): measures the matrix rate the device sustains, its clock under that load included,
 * before any operand is fetched -- the ceiling beside which the weight-gradient kernels are read.
 * d_sink (device, float[workgroups]) receives one value per workgroup; *flops (host, may be NULL)
 * the floating-point operations of the launch.  iters <= 2^24, workgroups <= 2^16 (SAMO_ERR_SIZE).
 * Not part of the method. */
samo_status samo_mfma_rate_probe(int64_t iters, float *d_sink, int32_t workgroups, double *flops,
                                 void *stream);

/* ---------------------------------------------------------------- tuning and testing aids
 * Process-wide knobs, set from the host; the entry points read no environment variable.  A knob
 * keeps its value until it is set again; SAMO_KNOB_DEFAULT as the value restores the built-in
 * choice.  Not needed for normal use: the defaults are the measured optima.
 *   SAMO_KNOB_OCC_TILE_STEP, _OCC_TILE_STEP32, _OCC_TILE_DECOMP, _OCC_TILE_C16 (workgroups) and
 *   SAMO_KNOB_OCC_FLAT_GATHER, _OCC_FLAT_STATS, _OCC_FLAT_STEP (waves)
 *                        resident per compute unit that a launch of that kind aims at; 0 = no cap.
 *   SAMO_KNOB_INDEX_SPIN_LIMIT  polls an index-build workgroup spends on a predecessor before it
 *                        gives up (default 2^20); 0 makes the give-up path reachable in tests.
 *   SAMO_KNOB_INDEX_PASSES  1, 2 or 4: forces the block size of the index build (64 KiB of mask per pass and
 *                        workgroup; default: 4 for launches with at least a dozen blocks of that size per
 *                        compute unit, else 2 or 1).
 *   SAMO_KNOB_WGRAD_TILE   128 or 256: forces the tile shape of the weight-gradient entries
 *                        (default: 128 x 128 for layers of at most 128 tiles of 256 x 256, which
 *                        would leave compute units idle, else 256 x 256 in whole rounds of the
 *                        compute units and 128 x 128 for a remainder of at most half a round).
 *   SAMO_KNOB_WGRAD_ROUND  test aid: the number of tiles taken as one round in that rule, in
 *                        place of the device's compute-unit count.
 *   SAMO_KNOB_TILE_COST    the weight of a plan's tiles in units of 1024 (6 .. 96; default 32, or 48 for a
 *                        model that keeps under 7 % of its elements; 48 there with an fp32 dense side).
 *                        Read by samo_plan_workspace_bytes and samo_plan_init: set it before both.
 * Returns SAMO_ERR_ARG for an unknown knob. */
enum {
    SAMO_KNOB_OCC_TILE_STEP = 0,
    SAMO_KNOB_OCC_TILE_STEP32 = 1,
    SAMO_KNOB_OCC_TILE_DECOMP = 2,
    SAMO_KNOB_OCC_TILE_C16 = 3,
    SAMO_KNOB_OCC_FLAT_GATHER = 4,
    SAMO_KNOB_OCC_FLAT_STATS = 5,
    SAMO_KNOB_OCC_FLAT_STEP = 6,
    SAMO_KNOB_INDEX_SPIN_LIMIT = 7,
    SAMO_KNOB_WGRAD_TILE = 8,
    SAMO_KNOB_WGRAD_ROUND = 9,
    SAMO_KNOB_INDEX_PASSES = 10,
    SAMO_KNOB_TILE_COST = 11,
    SAMO_KNOB_COUNT = 12
};
#define SAMO_KNOB_DEFAULT (-1)
samo_status samo_debug_set(int32_t knob, int32_t value);

#ifdef __cplusplus
}
#endif
#endif /* SAMO_H */
