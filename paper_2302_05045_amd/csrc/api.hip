// C ABI of libsamo: host-side argument validation, plan management, launches.
// Every entry point validates on the host first and enqueues only if all
// arguments are acceptable, so the error paths can be exercised without a GPU.
#include <atomic>
#include <cmath>
#include <cstring>

#include "common.h"

using namespace samo;

namespace samo {
namespace {
std::atomic<int> g_knobs[SAMO_KNOB_COUNT] = {};       // value + 1; 0 = built-in choice
}
int knob(int which, int dflt)
{
    const int v = g_knobs[which].load(std::memory_order_relaxed);
    return v > 0 ? v - 1 : dflt;
}
}  // namespace samo

namespace {

// Which arrays every layer of a plan provides (samo_plan::buffers).
enum : uint32_t {
    kHasP = 1u << 0, kHasM = 1u << 1, kHasV = 1u << 2, kHasW = 1u << 3, kHasG = 1u << 4, kHasGc = 1u << 5,
    kHasGc16 = 1u << 6, kHasW32 = 1u << 7, kHasG32 = 1u << 8, kHasAll = (1u << 9) - 1u,
    kPlanSegsShift = 16      // bits 16-23 of samo_plan::buffers: the most segments a tile of the plan holds
};
inline bool has(const samo_plan *plan, uint32_t bits) { return (plan->buffers & bits) == bits; }

// The static scratch array of the entry points that may not allocate: device memory that belongs
// to the library's code object, one copy per GPU at that GPU's own address.  In host code its name
// is only a handle for hipGetSymbolAddress; kernels get the resolved address as an argument.
constexpr size_t kStaticScratchBytes = 16u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices] = {};

// Number of compute units of the current device (looked up once per device; 256 if the query fails).
int compute_units()
{
    static std::atomic<int> cached[kMaxDevices] = {};
    int device = 0, n = 0;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) return 256;
    n = cached[device].load(std::memory_order_relaxed);
    if (n <= 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || n <= 0) n = 256;
        cached[device].store(n, std::memory_order_relaxed);
    }
    return n;
}

// Device address of `scratch` on the current device (looked up once per device, then cached).
hipError_t static_scratch(void **ptr)
{
    int device = 0;
    if (hipError_t e = hipGetDevice(&device)) return e;
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    void *p = g_scratch_ptr[device].load(std::memory_order_acquire);
    if (!p) {
        if (hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch))) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[device].store(p, std::memory_order_release);
    }
    *ptr = p;
    return hipSuccess;
}

constexpr int64_t kMaxN = 2147483647LL;   // the per-layer index is 32-bit (Section III-B)

inline bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }
inline samo_status hip_status(hipError_t e) { return e == hipSuccess ? SAMO_OK : SAMO_ERR_HIP; }
inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

// Tile records of a layer in a plan: one per segment of an unpruned layer; for a pruned layer as
// many as its total weight holds tiles of weight tile_cost.
int64_t tile_records(const samo_layer &L, int64_t tile_cost)
{
    const int64_t nseg = ceil_div(L.n, kSeg);
    if (nseg == 0 || !L.seg_ptr) return nseg;
    return ceil_div(kSegCost * nseg + kNnzCost * L.nnz, tile_cost);
}

samo_status check_sizes(int64_t n, int64_t nnz)
{
    if (n < 0 || n > kMaxN) return SAMO_ERR_SIZE;
    if (nnz < 0 || nnz > n) return SAMO_ERR_SIZE;
    return SAMO_OK;
}

samo_status check_scale(float s)
{
    return (std::isfinite(s) && s > 0.f) ? SAMO_OK : SAMO_ERR_ARG;
}

samo_status make_adam(const samo_adam_cfg *c, AdamK *k)
{
    if (!c) return SAMO_ERR_NULL;
    if (!std::isfinite(c->lr)) return SAMO_ERR_ARG;
    if (!(c->beta1 >= 0.f && c->beta1 < 1.f) || !(c->beta2 >= 0.f && c->beta2 < 1.f)) return SAMO_ERR_ARG;
    if (!(std::isfinite(c->eps) && c->eps > 0.f)) return SAMO_ERR_ARG;
    if (!(std::isfinite(c->weight_decay) && c->weight_decay >= 0.f)) return SAMO_ERR_ARG;
    if (c->step < 1) return SAMO_ERR_ARG;
    const double b1 = c->beta1, b2 = c->beta2;
    k->lr = c->lr;
    k->b1 = c->beta1;
    k->b2 = c->beta2;
    k->omb1 = (float)(1.0 - b1);
    k->omb2 = (float)(1.0 - b2);
    k->eps = c->eps;
    k->wd = c->weight_decay;
    k->rbc1 = (float)(1.0 / (1.0 - std::pow(b1, (double)c->step)));
    k->rbc2 = (float)(1.0 / (1.0 - std::pow(b2, (double)c->step)));
    k->l2 = (c->weight_decay != 0.f && !c->decoupled_wd) ? 1 : 0;
    k->decoupled = (c->weight_decay != 0.f && c->decoupled_wd) ? 1 : 0;
    return SAMO_OK;
}

// Index arguments of a layer: (idx, seg_ptr) both given (idx may be NULL when nnz == 0), or, where
// a dense layer is allowed, both NULL with nnz == n.
samo_status check_index_args(const int32_t *idx, const int32_t *seg_ptr, int64_t n, int64_t nnz, bool allow_dense)
{
    if (!idx && !seg_ptr) {
        if (!allow_dense) return SAMO_ERR_NULL;
        return nnz == n ? SAMO_OK : SAMO_ERR_SIZE;
    }
    if (!seg_ptr || (!idx && nnz > 0)) return SAMO_ERR_NULL;
    if (misaligned(idx) || misaligned(seg_ptr)) return SAMO_ERR_ALIGN;
    return SAMO_OK;
}

}  // namespace

extern "C" {

const char *samo_status_string(samo_status s)
{
    switch (s) {
    case SAMO_OK: return "ok";
    case SAMO_ERR_NULL: return "a required pointer is NULL";
    case SAMO_ERR_SIZE: return "size out of range (0 <= nnz <= n <= 2^31-1) or capacity too small";
    case SAMO_ERR_ARG: return "invalid hyper-parameter or loss scale";
    case SAMO_ERR_WORKSPACE: return "workspace missing or too small";
    case SAMO_ERR_ALIGN: return "pointer is not 16-byte aligned";
    case SAMO_ERR_INDEX: return "the index is not valid (build gave up, or not strictly ascending within the layer)";
    case SAMO_ERR_HIP: return "HIP runtime error";
    case SAMO_ERR_PLAN: return "plan lacks a buffer this entry point needs";
    default: return "unknown status";
    }
}

int32_t samo_abi_version(void) { return SAMO_ABI_VERSION; }

samo_status samo_init(void)
{
    int cus = 0;
    void *p = nullptr;
    if (wgrad_configure(&cus) != hipSuccess) return SAMO_ERR_HIP;
    return hip_status(static_scratch(&p));
}

samo_status samo_debug_set(int32_t which, int32_t value)
{
    if (which < 0 || which >= SAMO_KNOB_COUNT) return SAMO_ERR_ARG;
    g_knobs[which].store(value < 0 ? 0 : value + 1, std::memory_order_relaxed);
    return SAMO_OK;
}

samo_status samo_index_workspace_bytes(int64_t n, size_t *bytes)
{
    if (!bytes) return SAMO_ERR_NULL;
    if (n < 0 || n > kMaxN) return SAMO_ERR_SIZE;
    *bytes = (size_t)(ceil_div(n, kSeg) + 1) * sizeof(int32_t);
    return SAMO_OK;
}

int64_t samo_seg_ptr_len(int64_t n)
{
    if (n < 0 || n > kMaxN) return -1;
    return ceil_div(n, kSeg) + 1;
}

samo_status samo_build_index_batched(const samo_index_job *h_jobs, int32_t num_jobs, void *stream)
{
    if (num_jobs < 0) return SAMO_ERR_SIZE;
    if (num_jobs > 0 && !h_jobs) return SAMO_ERR_NULL;
    for (int32_t j = 0; j < num_jobs; ++j) {                      // validate everything before any launch
        const samo_index_job &J = h_jobs[j];
        if (J.n < 0 || J.n > kMaxN || J.idx_capacity < 0) return SAMO_ERR_SIZE;
        if ((!J.mask && J.n > 0) || !J.seg_ptr || !J.nnz || (!J.idx && J.idx_capacity > 0)) return SAMO_ERR_NULL;
        if (misaligned(J.mask) || misaligned(J.seg_ptr) || misaligned(J.idx) ||
            (reinterpret_cast<uintptr_t>(J.nnz) & 7u))
            return SAMO_ERR_ALIGN;
    }
    const int cus = compute_units();
    for (int32_t j0 = 0; j0 < num_jobs;) {
        IndexBatch batch;
        std::memset(&batch, 0, sizeof(batch));
        // testing aid: a tiny limit makes the give-up path (nnz = -1) reachable from the host
        batch.spin_limit = knob(SAMO_KNOB_INDEX_SPIN_LIMIT, kIndexSpinLimit);
        // the jobs of this launch (the grid stays within 2^31 - 1 workgroups whatever the block size),
        // then the block size the launch's volume of mask calls for
        int k = 0;
        int64_t bytes = 0, most = 0;
        for (; k < kIndexBatchJobs && j0 + k < num_jobs; ++k) {
            const int64_t w = index_job_workgroups(h_jobs[j0 + k].n, 1);
            if (k > 0 && most + w > kMaxN) break;
            most += w;
            bytes += h_jobs[j0 + k].n;
        }
        const int forced = knob(SAMO_KNOB_INDEX_PASSES, 0);
        batch.passes = (forced == 1 || forced == 2 || forced == 4) ? forced : index_passes_for(bytes, cus);
        batch.num = k;
        bool fill = false;
        int64_t wgs = 0;
        for (int i = 0; i < k; ++i) {
            const samo_index_job &J = h_jobs[j0 + i];
            const int64_t w = index_job_workgroups(J.n, batch.passes);
            batch.wg_start[i] = (int)wgs;
            batch.mask[i] = J.mask;
            batch.n[i] = J.n;
            batch.idx[i] = J.idx;
            batch.cap[i] = J.idx_capacity;
            batch.seg_ptr[i] = J.seg_ptr;
            batch.nnz[i] = J.nnz;
            fill |= J.idx_capacity > 0;
            if (w > 0) batch.ticket = J.nnz;
            wgs += w;
        }
        batch.wg_start[k] = (int)wgs;
        if (launch_index_batch(batch, fill, as_stream(stream)) != hipSuccess) return SAMO_ERR_HIP;
        j0 += k;
    }
    return SAMO_OK;
}

samo_status samo_count_nonzero(const uint8_t *d_mask, int64_t n, int32_t *d_seg_ptr, int64_t *d_nnz, void *stream)
{
    const samo_index_job job = {d_mask, n, nullptr, 0, d_seg_ptr, d_nnz};
    return samo_build_index_batched(&job, 1, stream);
}

samo_status samo_build_index(const uint8_t *d_mask, int64_t n, int32_t *d_idx, int64_t idx_capacity,
                             int32_t *d_seg_ptr, int64_t *d_nnz, void *stream)
{
    const samo_index_job job = {d_mask, n, d_idx, idx_capacity, d_seg_ptr, d_nnz};
    return samo_build_index_batched(&job, 1, stream);
}

samo_status samo_build_seg_ptr(const int32_t *d_idx, int64_t nnz, int64_t n, int32_t *d_seg_ptr, void *stream)
{
    if (samo_status s = check_sizes(n, nnz)) return s;
    if ((!d_idx && nnz > 0) || !d_seg_ptr) return SAMO_ERR_NULL;
    if (misaligned(d_idx) || misaligned(d_seg_ptr)) return SAMO_ERR_ALIGN;
    return hip_status(launch_seg_ptr_from_idx(d_idx, nnz, n, d_seg_ptr, as_stream(stream)));
}

samo_status samo_validate_index(const int32_t *d_idx, int64_t nnz, int64_t n, const int32_t *d_seg_ptr,
                                int32_t *d_ok, void *stream)
{
    if (samo_status s = check_sizes(n, nnz)) return s;
    if ((!d_idx && nnz > 0) || !d_ok) return SAMO_ERR_NULL;
    if (misaligned(d_idx) || misaligned(d_seg_ptr) || (reinterpret_cast<uintptr_t>(d_ok) & 3u)) return SAMO_ERR_ALIGN;
    return hip_status(launch_validate(d_idx, nnz, n, d_seg_ptr, d_ok, as_stream(stream)));
}

}  // extern "C"

namespace {

LaunchSet single(const samo_layer &L, int64_t wgs)
{
    LaunchSet ls;
    ls.one = L;
    ls.layers = nullptr;
    ls.recs = nullptr;
    ls.wgs = wgs;
    ls.segs_per_tile = 1;
    ls.keep = L.n > 0 ? (float)((double)L.nnz / (double)L.n) : 1.f;
    ls.max_segs = 1;
    return ls;
}

// Single-layer tile launch: every workgroup owns the same number of segments, chosen from the
// layer's average density (the per-region balance of a plan needs seg_ptr's contents).
LaunchSet single_tiles(const samo_layer &L)
{
    const int segs = single_layer_tile_segs(L.n, L.nnz, L.seg_ptr == nullptr, L.w32 != nullptr);
    LaunchSet ls = single(L, ceil_div(ceil_div(L.n, kSeg), segs));
    ls.segs_per_tile = segs;
    ls.max_segs = segs;
    return ls;
}

const GuardK kNoGuard = {nullptr, 0.f, 0};

samo_status make_sgd(const samo_sgd_cfg *c, OptK *k)
{
    if (!c) return SAMO_ERR_NULL;
    if (!std::isfinite(c->lr)) return SAMO_ERR_ARG;
    if (!(c->momentum >= 0.f && c->momentum < 1.f)) return SAMO_ERR_ARG;
    if (!(std::isfinite(c->weight_decay) && c->weight_decay >= 0.f)) return SAMO_ERR_ARG;
    std::memset(k, 0, sizeof(*k));
    k->sgd_lr = c->lr;
    k->sgd_mu = c->momentum;
    k->sgd_wd = c->weight_decay;
    return SAMO_OK;
}

samo_status make_adam_opt(const samo_adam_cfg *c, OptK *k)
{
    std::memset(k, 0, sizeof(*k));
    return make_adam(c, &k->adam);
}

samo_status make_guard(const samo_step_guard *g, GuardK *out)
{
    *out = kNoGuard;
    if (!g) return SAMO_OK;
    if (!(g->max_grad_norm == g->max_grad_norm) || std::isinf(g->max_grad_norm)) return SAMO_ERR_ARG;
    const bool used = g->max_grad_norm > 0.f || g->skip_on_nonfinite != 0;
    if (used && !g->d_stats) return SAMO_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(g->d_stats) & 7u) return SAMO_ERR_ALIGN;
    if (used) {
        out->stats = g->d_stats;
        out->max_norm = g->max_grad_norm;
        out->skip = g->skip_on_nonfinite != 0;
    }
    return SAMO_OK;
}

// Common argument checks of the single-layer step entries (dense layers allowed).
samo_status check_step_args(const void *grad, uint16_t *w, int64_t n, const int32_t *idx, const int32_t *seg_ptr,
                            int64_t nnz, const float *p, const float *m, const float *v, bool need_v,
                            float inv_loss_scale)
{
    if (samo_status s = check_sizes(n, nnz)) return s;
    if (samo_status s = check_index_args(idx, seg_ptr, n, nnz, /*allow_dense=*/true)) return s;
    if (n > 0 && !w) return SAMO_ERR_NULL;
    if (nnz > 0 && (!grad || !p || !m || (need_v && !v))) return SAMO_ERR_NULL;
    if (misaligned(grad) || misaligned(w) || misaligned(p) || misaligned(m) || misaligned(v)) return SAMO_ERR_ALIGN;
    return check_scale(inv_loss_scale);
}

}  // namespace

extern "C" {

samo_status samo_decompress(const float *d_p, const int32_t *d_idx, const int32_t *d_seg_ptr, int64_t nnz,
                            uint16_t *d_w, int64_t n, void *stream)
{
    if (samo_status s = check_sizes(n, nnz)) return s;
    if (samo_status s = check_index_args(d_idx, d_seg_ptr, n, nnz, /*allow_dense=*/true)) return s;
    if ((!d_p && nnz > 0) || (!d_w && n > 0)) return SAMO_ERR_NULL;
    if (misaligned(d_p) || misaligned(d_w)) return SAMO_ERR_ALIGN;
    samo_layer L = {n, nnz, d_idx, d_seg_ptr, const_cast<float *>(d_p), nullptr, nullptr, d_w, nullptr, nullptr,
                    nullptr, nullptr, nullptr};
    OptK k;
    std::memset(&k, 0, sizeof(k));
    return hip_status(launch_tile(kModeDecompress, kGradDense, kOptAdam, single_tiles(L), 1.f, k,
                                  kNoGuard, as_stream(stream)));
}

samo_status samo_gather_grads(const uint16_t *d_g, int64_t n, const int32_t *d_idx, int64_t nnz,
                              float inv_loss_scale, float *d_gc, void *stream)
{
    if (samo_status s = check_sizes(n, nnz)) return s;
    if (!d_idx && nnz > 0 && nnz != n) return SAMO_ERR_NULL;      /* NULL idx = dense layer */
    if (nnz > 0 && (!d_g || !d_gc)) return SAMO_ERR_NULL;
    if (misaligned(d_g) || misaligned(d_idx) || misaligned(d_gc)) return SAMO_ERR_ALIGN;
    if (samo_status s = check_scale(inv_loss_scale)) return s;
    samo_layer L = {n, nnz, d_idx, nullptr, nullptr, nullptr, nullptr, nullptr, d_g, d_gc, nullptr, nullptr, nullptr};
    return hip_status(launch_gather(kOutF32, kGradDense, single(L, ceil_div(nnz, kChunk)), inv_loss_scale, 0, nullptr,
                                    as_stream(stream)));
}

samo_status samo_gather_grads_fp16(const uint16_t *d_g, int64_t n, const int32_t *d_idx, int64_t nnz,
                                   uint16_t *d_gc16, int32_t accumulate, void *stream)
{
    if (samo_status s = check_sizes(n, nnz)) return s;
    if (!d_idx && nnz > 0 && nnz != n) return SAMO_ERR_NULL;
    if (nnz > 0 && (!d_g || !d_gc16)) return SAMO_ERR_NULL;
    if (misaligned(d_g) || misaligned(d_idx) || misaligned(d_gc16)) return SAMO_ERR_ALIGN;
    samo_layer L = {n, nnz, d_idx, nullptr, nullptr, nullptr, nullptr, nullptr, d_g, nullptr, d_gc16, nullptr, nullptr};
    return hip_status(launch_gather(kOutF16, kGradDense, single(L, ceil_div(nnz, kChunk)), 1.f, accumulate != 0,
                                    nullptr, as_stream(stream)));
}

namespace {
samo_status check_wgrad(const void *d_dy, const void *d_x, int64_t tokens, int64_t out, int64_t in,
                        const int32_t *d_idx, const int32_t *d_seg_ptr, int64_t nnz, const void *d_out)
{
    if (tokens < 0 || tokens > kMaxN || out <= 0 || in <= 0 || out > kMaxN || in > kMaxN) return SAMO_ERR_SIZE;
    if ((out & 7) || (in & 7)) return SAMO_ERR_SIZE;
    if (out > (1 << 24) || in > (1 << 24)) return SAMO_ERR_SIZE;   // 32-bit byte offsets within a stage of 32 tokens
    if (out > kMaxN / in) return SAMO_ERR_SIZE;
    if (samo_status s = check_sizes(out * in, nnz)) return s;
    if (nnz == 0) return SAMO_OK;
    if (!d_out || (tokens > 0 && (!d_dy || !d_x))) return SAMO_ERR_NULL;
    if (!d_idx && nnz != out * in) return SAMO_ERR_NULL;
    if (d_idx && !d_seg_ptr) return SAMO_ERR_NULL;
    if (misaligned(d_dy) || misaligned(d_x) || misaligned(d_idx) || misaligned(d_out)) return SAMO_ERR_ALIGN;
    return SAMO_OK;
}
}  // namespace

namespace {
samo_status wgrad_batched(int out_kind, int32_t count, const samo_wgrad_job *h_jobs, float inv_scale, int accumulate,
                          void *stream)
{
    if (count < 0 || count > SAMO_WGRAD_MAX_JOBS) return SAMO_ERR_SIZE;
    if (count > 0 && !h_jobs) return SAMO_ERR_NULL;
    WgradJob jobs[SAMO_WGRAD_MAX_JOBS];
    for (int j = 0; j < count; ++j) {
        const samo_wgrad_job &h = h_jobs[j];
        if (samo_status s = check_wgrad(h.d_dy, h.d_x, h.tokens, h.out, h.in, h.d_idx, h.d_seg_ptr, h.nnz, h.d_gc)) return s;
        jobs[j] = {reinterpret_cast<const _Float16 *>(h.d_dy), reinterpret_cast<const _Float16 *>(h.d_x), h.tokens,
                   (int)h.out, (int)h.in, h.d_idx, h.d_seg_ptr, h.nnz, h.d_gc};
    }
    return hip_status(launch_wgrad(out_kind, jobs, count, inv_scale, accumulate, as_stream(stream)));
}
}  // namespace

samo_status samo_wgrad_gather(const uint16_t *d_dy, const uint16_t *d_x, int64_t tokens, int64_t out, int64_t in,
                              const int32_t *d_idx, const int32_t *d_seg_ptr, int64_t nnz, float inv_loss_scale,
                              float *d_gc, void *stream)
{
    const samo_wgrad_job job = {d_dy, d_x, tokens, out, in, d_idx, d_seg_ptr, nnz, d_gc};
    return samo_wgrad_gather_batched(1, &job, inv_loss_scale, stream);
}

samo_status samo_wgrad_gather_fp16(const uint16_t *d_dy, const uint16_t *d_x, int64_t tokens, int64_t out, int64_t in,
                                   const int32_t *d_idx, const int32_t *d_seg_ptr, int64_t nnz, uint16_t *d_gc16,
                                   int32_t accumulate, void *stream)
{
    const samo_wgrad_job job = {d_dy, d_x, tokens, out, in, d_idx, d_seg_ptr, nnz, d_gc16};
    return samo_wgrad_gather_fp16_batched(1, &job, accumulate, stream);
}

samo_status samo_wgrad_gather_batched(int32_t count, const samo_wgrad_job *h_jobs, float inv_loss_scale, void *stream)
{
    if (samo_status s = check_scale(inv_loss_scale)) return s;
    return wgrad_batched(kOutF32, count, h_jobs, inv_loss_scale, 0, stream);
}

samo_status samo_wgrad_gather_fp16_batched(int32_t count, const samo_wgrad_job *h_jobs, int32_t accumulate, void *stream)
{
    return wgrad_batched(kOutF16, count, h_jobs, 1.f, accumulate != 0, stream);
}

samo_status samo_adam_step(float *d_p, float *d_m, float *d_v, const float *d_gc, int64_t nnz,
                           const samo_adam_cfg *h_cfg, void *stream)
{
    if (nnz < 0 || nnz > kMaxN) return SAMO_ERR_SIZE;
    if (nnz > 0 && (!d_p || !d_m || !d_v || !d_gc)) return SAMO_ERR_NULL;
    if (misaligned(d_p) || misaligned(d_m) || misaligned(d_v) || misaligned(d_gc)) return SAMO_ERR_ALIGN;
    OptK k;
    if (samo_status s = make_adam_opt(h_cfg, &k)) return s;
    samo_layer L = {nnz, nnz, nullptr, nullptr, d_p, d_m, d_v, nullptr, nullptr, const_cast<float *>(d_gc), nullptr, nullptr, nullptr};
    return hip_status(launch_flat_step(kOptAdam, single(L, ceil_div(nnz, kChunk)), k, kNoGuard, as_stream(stream)));
}

samo_status samo_sgd_step(float *d_p, float *d_buf, const float *d_gc, int64_t nnz, const samo_sgd_cfg *h_cfg,
                          void *stream)
{
    if (nnz < 0 || nnz > kMaxN) return SAMO_ERR_SIZE;
    if (nnz > 0 && (!d_p || !d_buf || !d_gc)) return SAMO_ERR_NULL;
    if (misaligned(d_p) || misaligned(d_buf) || misaligned(d_gc)) return SAMO_ERR_ALIGN;
    OptK k;
    if (samo_status s = make_sgd(h_cfg, &k)) return s;
    samo_layer L = {nnz, nnz, nullptr, nullptr, d_p, d_buf, nullptr, nullptr, nullptr, const_cast<float *>(d_gc),
                    nullptr, nullptr, nullptr};
    return hip_status(launch_flat_step(kOptSgd, single(L, ceil_div(nnz, kChunk)), k, kNoGuard, as_stream(stream)));
}

samo_status samo_fused_step(const uint16_t *d_g, uint16_t *d_w, int64_t n, const int32_t *d_idx,
                            const int32_t *d_seg_ptr, int64_t nnz, float *d_p, float *d_m, float *d_v,
                            float inv_loss_scale, const samo_adam_cfg *h_cfg, void *stream)
{
    if (samo_status s = check_step_args(d_g, d_w, n, d_idx, d_seg_ptr, nnz, d_p, d_m, d_v, true, inv_loss_scale))
        return s;
    if (n > 0 && !d_g) return SAMO_ERR_NULL;
    OptK k;
    if (samo_status s = make_adam_opt(h_cfg, &k)) return s;
    samo_layer L = {n, nnz, d_idx, d_seg_ptr, d_p, d_m, d_v, d_w, d_g, nullptr, nullptr, nullptr, nullptr};
    return hip_status(launch_tile(kModeStep, kGradDense, kOptAdam, single_tiles(L), inv_loss_scale, k,
                                  kNoGuard, as_stream(stream)));
}

samo_status samo_adam_expand_step(const uint16_t *d_gc16, uint16_t *d_w, int64_t n, const int32_t *d_idx,
                                  const int32_t *d_seg_ptr, int64_t nnz, float *d_p, float *d_m, float *d_v,
                                  float inv_loss_scale, const samo_adam_cfg *h_cfg, void *stream)
{
    if (samo_status s = check_step_args(d_gc16, d_w, n, d_idx, d_seg_ptr, nnz, d_p, d_m, d_v, true, inv_loss_scale))
        return s;
    OptK k;
    if (samo_status s = make_adam_opt(h_cfg, &k)) return s;
    samo_layer L = {n, nnz, d_idx, d_seg_ptr, d_p, d_m, d_v, d_w, nullptr, nullptr, const_cast<uint16_t *>(d_gc16), nullptr, nullptr};
    return hip_status(launch_tile(kModeStep, kGradC16, kOptAdam, single_tiles(L), inv_loss_scale, k,
                                  kNoGuard, as_stream(stream)));
}

samo_status samo_fused_sgd_step(const uint16_t *d_g, uint16_t *d_w, int64_t n, const int32_t *d_idx,
                                const int32_t *d_seg_ptr, int64_t nnz, float *d_p, float *d_buf,
                                float inv_loss_scale, const samo_sgd_cfg *h_cfg, void *stream)
{
    if (samo_status s = check_step_args(d_g, d_w, n, d_idx, d_seg_ptr, nnz, d_p, d_buf, nullptr, false,
                                        inv_loss_scale))
        return s;
    if (n > 0 && !d_g) return SAMO_ERR_NULL;
    OptK k;
    if (samo_status s = make_sgd(h_cfg, &k)) return s;
    samo_layer L = {n, nnz, d_idx, d_seg_ptr, d_p, d_buf, nullptr, d_w, d_g, nullptr, nullptr, nullptr, nullptr};
    return hip_status(launch_tile(kModeStep, kGradDense, kOptSgd, single_tiles(L), inv_loss_scale, k,
                                  kNoGuard, as_stream(stream)));
}

// ------------------------------------------------------------------------------ plan
}  // extern "C"

namespace {

inline size_t round_up_256(size_t x) { return (x + 255u) & ~(size_t)255u; }

// Sizes of a plan's tables; validates the descriptors when `check` is set.
struct PlanSizes {
    int64_t ntiles = 0, nchunks = 0, n_total = 0, nnz_total = 0, tile_cost = kTileCost;
    uint32_t buffers = kHasAll;
    size_t off_tile_start = 0, off_chunk_start = 0, off_tiles = 0, off_chunks = 0, bytes = 0;
};

samo_status plan_sizes(const samo_layer *h_layers, int32_t num_layers, bool check, PlanSizes *out)
{
    if (num_layers < 0) return SAMO_ERR_SIZE;
    if (num_layers > 0 && !h_layers) return SAMO_ERR_NULL;
    PlanSizes z;
    for (int32_t l = 0; l < num_layers; ++l) {
        const samo_layer &L = h_layers[l];
        if (samo_status s = check_sizes(L.n, L.nnz)) return s;
        if (check) {
            if (samo_status s = check_index_args(L.idx, L.seg_ptr, L.n, L.nnz, /*allow_dense=*/true)) return s;
            if (!L.p && !L.w32 && L.nnz > 0) return SAMO_ERR_NULL;      // parameters in one form at least
            if (misaligned(L.p) || misaligned(L.m) || misaligned(L.v) || misaligned(L.w) || misaligned(L.g) ||
                misaligned(L.gc) || misaligned(L.gc16) || misaligned(L.w32) || misaligned(L.g32))
                return SAMO_ERR_ALIGN;
            if (L.nnz > 0) {
                if (!L.p) z.buffers &= ~kHasP;
                if (!L.m) z.buffers &= ~kHasM;
                if (!L.v) z.buffers &= ~kHasV;
                if (!L.gc) z.buffers &= ~kHasGc;
                if (!L.gc16) z.buffers &= ~kHasGc16;
            }
            if (L.n > 0) {
                if (!L.w) z.buffers &= ~kHasW;
                if (!L.g) z.buffers &= ~kHasG;
                if (!L.w32) z.buffers &= ~kHasW32;
                if (!L.g32) z.buffers &= ~kHasG32;
            }
        }
        z.n_total += L.n;
        z.nnz_total += L.nnz;
        z.nchunks += ceil_div(L.nnz, kChunk);
    }
    // one tile weight for the whole plan, by its kept fraction and the width of its dense side; when only
    // the sizes are asked for (the arrays need not be known yet), the lighter of the two: more records
    z.tile_cost = tile_cost_for(z.n_total, z.nnz_total, (z.buffers & kHasW32) != 0);
    if (!check) {
        const int64_t other = tile_cost_for(z.n_total, z.nnz_total, false);
        if (other < z.tile_cost) z.tile_cost = other;
    }
    for (int32_t l = 0; l < num_layers; ++l) z.ntiles += tile_records(h_layers[l], z.tile_cost);
    if (z.ntiles > kMaxN || z.nchunks > kMaxN) return SAMO_ERR_SIZE;
    size_t at = round_up_256((size_t)num_layers * sizeof(samo_layer));
    z.off_tile_start = at;
    at += round_up_256(((size_t)num_layers + 1) * sizeof(int64_t));
    z.off_chunk_start = at;
    at += round_up_256(((size_t)num_layers + 1) * sizeof(int64_t));
    z.off_tiles = at;
    at += round_up_256((size_t)z.ntiles * sizeof(WgRec));
    z.off_chunks = at;
    at += round_up_256((size_t)z.nchunks * sizeof(WgRec));
    z.bytes = at;
    *out = z;
    return SAMO_OK;
}

}  // namespace

extern "C" {

samo_status samo_plan_workspace_bytes(const samo_layer *h_layers, int32_t num_layers, size_t *bytes)
{
    if (!bytes) return SAMO_ERR_NULL;
    PlanSizes z;
    if (samo_status s = plan_sizes(h_layers, num_layers, /*check=*/false, &z)) return s;
    *bytes = z.bytes;
    return SAMO_OK;
}

samo_status samo_plan_init(const samo_layer *h_layers, int32_t num_layers, void *d_workspace, size_t workspace_bytes,
                           void *stream, samo_plan *plan)
{
    if (!plan) return SAMO_ERR_NULL;
    PlanSizes z;
    if (samo_status s = plan_sizes(h_layers, num_layers, /*check=*/true, &z)) return s;
    if (!d_workspace || workspace_bytes < z.bytes) return SAMO_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(d_workspace) & 255u) return SAMO_ERR_ALIGN;

    unsigned char *ws = reinterpret_cast<unsigned char *>(d_workspace);
    PlanTables t;
    t.layers = reinterpret_cast<samo_layer *>(ws);
    t.tile_start = reinterpret_cast<int64_t *>(ws + z.off_tile_start);
    t.chunk_start = reinterpret_cast<int64_t *>(ws + z.off_chunk_start);
    t.tiles = reinterpret_cast<WgRec *>(ws + z.off_tiles);
    t.chunks = reinterpret_cast<WgRec *>(ws + z.off_chunks);

    // the layer table, kPlanBatchLayers descriptors per launch (a plan without layers still gets
    // its two start entries)
    int64_t tile_at = 0, chunk_at = 0;
    int32_t l = 0;
    do {
        PlanBatch b;
        std::memset(&b, 0, sizeof(b));
        b.first = l;
        int k = 0;
        for (; k < kPlanBatchLayers && l < num_layers; ++k, ++l) {
            b.layer[k] = h_layers[l];
            b.tile_start[k] = tile_at;
            b.chunk_start[k] = chunk_at;
            tile_at += tile_records(h_layers[l], z.tile_cost);
            chunk_at += ceil_div(h_layers[l].nnz, kChunk);
        }
        b.count = k;
        b.tile_start[k] = tile_at;
        b.chunk_start[k] = chunk_at;
        if (launch_plan_write(b, t, as_stream(stream)) != hipSuccess) return SAMO_ERR_HIP;
    } while (l < num_layers);
    if (launch_plan_records(t, num_layers, z.ntiles, z.nchunks, z.tile_cost, as_stream(stream)) != hipSuccess) return SAMO_ERR_HIP;

    plan->d_layers = t.layers;
    plan->d_tiles = t.tiles;
    plan->d_chunks = t.chunks;
    plan->num_tiles = z.ntiles;
    plan->num_chunks = z.nchunks;
    plan->n_total = z.n_total;
    plan->nnz_total = z.nnz_total;
    plan->num_layers = num_layers;
    plan->buffers = z.buffers | ((uint32_t)tile_cost_segs(z.tile_cost) << kPlanSegsShift);
    return SAMO_OK;
}

samo_status samo_plan_stats_workspace_bytes(const samo_plan *plan, size_t *bytes)
{
    if (!plan || !bytes) return SAMO_ERR_NULL;
    *bytes = (size_t)stats_workspace_partials(plan->num_chunks) * sizeof(StatPartial);
    return SAMO_OK;
}

}  // extern "C"

namespace {

LaunchSet tiles_of(const samo_plan *plan)
{
    LaunchSet ls;
    std::memset(&ls, 0, sizeof(ls));
    ls.layers = reinterpret_cast<const samo_layer *>(plan->d_layers);
    ls.recs = reinterpret_cast<const WgRec *>(plan->d_tiles);
    ls.wgs = plan->num_tiles;
    ls.segs_per_tile = 1;
    ls.keep = plan->n_total > 0 ? (float)((double)plan->nnz_total / (double)plan->n_total) : 1.f;
    ls.max_segs = (int)((plan->buffers >> kPlanSegsShift) & 0xffu);     // as samo_plan_init cut the tiles (checked at launch)
    return ls;
}

LaunchSet chunks_of(const samo_plan *plan)
{
    LaunchSet ls;
    std::memset(&ls, 0, sizeof(ls));
    ls.layers = reinterpret_cast<const samo_layer *>(plan->d_layers);
    ls.recs = reinterpret_cast<const WgRec *>(plan->d_chunks);
    ls.wgs = plan->num_chunks;
    ls.segs_per_tile = 1;
    ls.keep = plan->n_total > 0 ? (float)((double)plan->nnz_total / (double)plan->n_total) : 1.f;
    return ls;
}

// Workspace check of the entries that can reduce gradient statistics.
samo_status check_stats_args(const samo_plan *plan, const samo_grad_stats *d_stats, const void *ws, size_t ws_bytes)
{
    if (!d_stats) return SAMO_OK;
    size_t need = 0;
    samo_plan_stats_workspace_bytes(plan, &need);
    if (!ws || ws_bytes < need) return SAMO_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(d_stats) & 7u) || misaligned(ws)) return SAMO_ERR_ALIGN;
    return SAMO_OK;
}

// Gather-type launch over the plan's chunks, followed by the reduction of the partials.
samo_status run_gather(const samo_plan *plan, int out, int src, float inv_scale, int accumulate,
                       samo_grad_stats *d_stats, void *ws, hipStream_t s)
{
    StatPartial *partials = d_stats ? reinterpret_cast<StatPartial *>(ws) : nullptr;
    if (launch_gather(out, src, chunks_of(plan), inv_scale, accumulate, partials, s) != hipSuccess)
        return SAMO_ERR_HIP;
    if (d_stats) return hip_status(launch_stats_finalize(partials, plan->num_chunks, d_stats, s));
    return SAMO_OK;
}

}  // namespace

extern "C" {

samo_status samo_decompress_batched(const samo_plan *plan, void *stream)
{
    if (!plan) return SAMO_ERR_NULL;
    if (!has(plan, kHasW | kHasP)) return SAMO_ERR_PLAN;
    OptK k;
    std::memset(&k, 0, sizeof(k));
    return hip_status(launch_tile(kModeDecompress, kGradDense, kOptAdam, tiles_of(plan), 1.f, k, kNoGuard,
                                  as_stream(stream)));
}

samo_status samo_gather_batched(const samo_plan *plan, float inv_loss_scale, samo_grad_stats *d_stats,
                                void *d_workspace, size_t workspace_bytes, void *stream)
{
    if (!plan) return SAMO_ERR_NULL;
    if (!has(plan, kHasG | kHasGc)) return SAMO_ERR_PLAN;
    if (samo_status s = check_scale(inv_loss_scale)) return s;
    if (samo_status s = check_stats_args(plan, d_stats, d_workspace, workspace_bytes)) return s;
    return run_gather(plan, kOutF32, kGradDense, inv_loss_scale, 0, d_stats, d_workspace, as_stream(stream));
}

samo_status samo_gather_fp16_batched(const samo_plan *plan, int32_t accumulate, float inv_loss_scale,
                                     samo_grad_stats *d_stats, void *d_workspace, size_t workspace_bytes,
                                     void *stream)
{
    if (!plan) return SAMO_ERR_NULL;
    if (!has(plan, kHasG | kHasGc16)) return SAMO_ERR_PLAN;
    if (samo_status s = check_scale(inv_loss_scale)) return s;
    if (samo_status s = check_stats_args(plan, d_stats, d_workspace, workspace_bytes)) return s;
    return run_gather(plan, kOutF16, kGradDense, inv_loss_scale, accumulate != 0, d_stats, d_workspace,
                      as_stream(stream));
}

samo_status samo_grad_stats_batched(const samo_plan *plan, int32_t source, float inv_loss_scale,
                                    samo_grad_stats *d_stats, void *d_workspace, size_t workspace_bytes,
                                    void *stream)
{
    if (!plan || !d_stats) return SAMO_ERR_NULL;
    if (source < 0 || source > 3) return SAMO_ERR_ARG;
    if ((source == kGradDense && !has(plan, kHasG)) || (source == kGradC16 && !has(plan, kHasGc16)) ||
        (source == kGradC32 && !has(plan, kHasGc)) || (source == kGradDense32 && !has(plan, kHasG32)))
        return SAMO_ERR_PLAN;
    if (samo_status s = check_scale(inv_loss_scale)) return s;
    if (samo_status s = check_stats_args(plan, d_stats, d_workspace, workspace_bytes)) return s;
    return run_gather(plan, kOutNone, source, inv_loss_scale, 0, d_stats, d_workspace, as_stream(stream));
}

size_t samo_static_scratch_bytes(void) { return kStaticScratchBytes; }

samo_status samo_grad_stats_batched_static(const samo_plan *plan, int32_t source, float inv_loss_scale,
                                           samo_grad_stats *d_stats, void *stream)
{
    if (!plan || !d_stats) return SAMO_ERR_NULL;
    size_t need = 0;
    samo_plan_stats_workspace_bytes(plan, &need);
    if (need > kStaticScratchBytes) return SAMO_ERR_SIZE;      // checked first: the caller can fall back to its own workspace
    void *ws = nullptr;
    if (static_scratch(&ws) != hipSuccess) return SAMO_ERR_HIP;
    // every partial the reduction reads is written by this call's own launches first: nothing to clear
    return samo_grad_stats_batched(plan, source, inv_loss_scale, d_stats, ws, kStaticScratchBytes, stream);
}

samo_status samo_adam_batched(const samo_plan *plan, const samo_adam_cfg *h_cfg, const samo_step_guard *h_guard,
                              void *stream)
{
    if (!plan) return SAMO_ERR_NULL;
    if (!has(plan, kHasP | kHasM | kHasV | kHasGc)) return SAMO_ERR_PLAN;
    OptK k;
    GuardK guard;
    if (samo_status s = make_adam_opt(h_cfg, &k)) return s;
    if (samo_status s = make_guard(h_guard, &guard)) return s;
    return hip_status(launch_flat_step(kOptAdam, chunks_of(plan), k, guard, as_stream(stream)));
}

samo_status samo_fused_step_batched(const samo_plan *plan, float inv_loss_scale, const samo_adam_cfg *h_cfg,
                                    const samo_step_guard *h_guard, void *stream)
{
    if (!plan) return SAMO_ERR_NULL;
    if (!has(plan, kHasP | kHasM | kHasV | kHasW | kHasG)) return SAMO_ERR_PLAN;
    if (samo_status s = check_scale(inv_loss_scale)) return s;
    OptK k;
    GuardK guard;
    if (samo_status s = make_adam_opt(h_cfg, &k)) return s;
    if (samo_status s = make_guard(h_guard, &guard)) return s;
    return hip_status(launch_tile(kModeStep, kGradDense, kOptAdam, tiles_of(plan), inv_loss_scale, k, guard,
                                  as_stream(stream)));
}

samo_status samo_adam_expand_batched(const samo_plan *plan, float inv_loss_scale, const samo_adam_cfg *h_cfg,
                                     const samo_step_guard *h_guard, void *stream)
{
    if (!plan) return SAMO_ERR_NULL;
    if (!has(plan, kHasP | kHasM | kHasV | kHasW | kHasGc16)) return SAMO_ERR_PLAN;
    if (samo_status s = check_scale(inv_loss_scale)) return s;
    OptK k;
    GuardK guard;
    if (samo_status s = make_adam_opt(h_cfg, &k)) return s;
    if (samo_status s = make_guard(h_guard, &guard)) return s;
    return hip_status(launch_tile(kModeStep, kGradC16, kOptAdam, tiles_of(plan), inv_loss_scale, k, guard,
                                  as_stream(stream)));
}

samo_status samo_fused_sgd_step_batched(const samo_plan *plan, float inv_loss_scale, const samo_sgd_cfg *h_cfg,
                                        const samo_step_guard *h_guard, void *stream)
{
    if (!plan) return SAMO_ERR_NULL;
    if (!has(plan, kHasP | kHasM | kHasW | kHasG)) return SAMO_ERR_PLAN;
    if (samo_status s = check_scale(inv_loss_scale)) return s;
    OptK k;
    GuardK guard;
    if (samo_status s = make_sgd(h_cfg, &k)) return s;
    if (samo_status s = make_guard(h_guard, &guard)) return s;
    return hip_status(launch_tile(kModeStep, kGradDense, kOptSgd, tiles_of(plan), inv_loss_scale, k, guard,
                                  as_stream(stream)));
}

samo_status samo_fused_step_fp32(const float *d_g32, float *d_w32, int64_t n, const int32_t *d_idx,
                                 const int32_t *d_seg_ptr, int64_t nnz, float *d_m, float *d_v, float grad_factor,
                                 const samo_adam_cfg *h_cfg, void *stream)
{
    if (samo_status s = check_sizes(n, nnz)) return s;
    if (samo_status s = check_index_args(d_idx, d_seg_ptr, n, nnz, /*allow_dense=*/true)) return s;
    if (n > 0 && (!d_w32 || !d_g32)) return SAMO_ERR_NULL;
    if (nnz > 0 && (!d_m || !d_v)) return SAMO_ERR_NULL;
    if (misaligned(d_g32) || misaligned(d_w32) || misaligned(d_m) || misaligned(d_v)) return SAMO_ERR_ALIGN;
    if (samo_status s = check_scale(grad_factor)) return s;
    OptK k;
    if (samo_status s = make_adam_opt(h_cfg, &k)) return s;
    samo_layer L;
    std::memset(&L, 0, sizeof(L));
    L.n = n;
    L.nnz = nnz;
    L.idx = d_idx;
    L.seg_ptr = d_seg_ptr;
    L.m = d_m;
    L.v = d_v;
    L.w32 = d_w32;
    L.g32 = d_g32;
    return hip_status(launch_tile_fp32(single_tiles(L), grad_factor, k, kNoGuard, as_stream(stream)));
}

samo_status samo_fused_step_fp32_batched(const samo_plan *plan, float grad_factor, const samo_adam_cfg *h_cfg,
                                         const samo_step_guard *h_guard, void *stream)
{
    if (!plan) return SAMO_ERR_NULL;
    if (!has(plan, kHasM | kHasV | kHasW32 | kHasG32)) return SAMO_ERR_PLAN;
    if (samo_status s = check_scale(grad_factor)) return s;
    OptK k;
    GuardK guard;
    if (samo_status s = make_adam_opt(h_cfg, &k)) return s;
    if (samo_status s = make_guard(h_guard, &guard)) return s;
    return hip_status(launch_tile_fp32(tiles_of(plan), grad_factor, k, guard, as_stream(stream)));
}

samo_status samo_memory_model(int64_t n_total, int64_t nnz_total, int64_t *paper_default, int64_t *paper_samo,
                              int64_t *resident)
{
    if (n_total < 0 || nnz_total < 0 || nnz_total > n_total) return SAMO_ERR_SIZE;
    if (n_total > (INT64_MAX / 64)) return SAMO_ERR_SIZE;
    if (paper_default) *paper_default = 20 * n_total;
    if (paper_samo) *paper_samo = 24 * nnz_total + 2 * n_total;
    if (resident) *resident = 16 * nnz_total + 2 * n_total;
    return SAMO_OK;
}

samo_status samo_stream_copy(void *d_dst, const void *d_src, int64_t bytes, void *stream)
{
    if (bytes < 0 || (bytes & 15)) return SAMO_ERR_SIZE;
    if (bytes > 0 && (!d_dst || !d_src)) return SAMO_ERR_NULL;
    if (misaligned(d_dst) || misaligned(d_src)) return SAMO_ERR_ALIGN;
    return hip_status(launch_copy(d_dst, d_src, bytes, as_stream(stream)));
}

samo_status samo_mfma_rate_probe(int64_t iters, float *d_sink, int32_t workgroups, double *flops, void *stream)
{
    if (iters < 0 || iters > (1 << 24) || workgroups < 0 || workgroups > (1 << 16)) return SAMO_ERR_SIZE;
    if (workgroups > 0 && !d_sink) return SAMO_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(d_sink) & 3u) return SAMO_ERR_ALIGN;
    if (flops) *flops = 2.0 * 32 * 32 * 16 * 8 * kMfmaRateWaves * (double)iters * (double)workgroups;
    return hip_status(launch_mfma_rate(iters, d_sink, workgroups, as_stream(stream)));
}

}  // extern "C"
