// Expansion, gradient compression, optimizers on the compressed state and the fused optimizer
// phase (Section III-C of the paper) as HBM-streaming kernels for gfx950.
//
// Dense side (fp16 w and g, N elements): a workgroup owns a tile, a run of whole 1024-element
// segments of one layer chosen so that every workgroup moves about the same number of bytes.
// The new fp16 weights of the tile are assembled in LDS — zero filled, then the kept values
// dropped in at their tile-relative positions — and leave as whole 16-byte non-temporal stores,
// so HBM never sees a partial-line write and the explicit zeros of the pruned positions cost no
// extra pass.
// Compressed side (idx, p, m, v, gc, gc16; nnz elements): the tile's slice is
// [seg_ptr[first segment], seg_ptr[last segment + 1]); consecutive lanes take consecutive
// compressed elements, so every access is a contiguous run.  Gradients of the dense buffer are
// read at the kept positions only; with ascending indices the lanes of a wave fall into a
// handful of neighbouring cache lines.
//
// There is no matrix contraction anywhere on this path: it is bound by HBM bandwidth, and each
// byte is touched once.
#include <cfloat>
#include <cstdlib>

#include "common.h"

namespace samo {
namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float half_bits_to_float(uint16_t h)
{
    return (float)__builtin_bit_cast(_Float16, h);          // exact, subnormals honoured
}

// fp32 -> fp16, round to nearest even.  The empty asm makes x opaque, so the conversion always
// starts from the fp32 value that is also stored as the master parameter; without it the compiler
// folds the last fma of the update and this conversion into one v_fma_mixlo_f16, which rounds
// the exact fma result once to fp16 and so differs from fp16(fp32(p)) on double-rounding cases.
__device__ __forceinline__ uint16_t float_to_half_bits(float x)
{
    asm("" : "+v"(x));
    return __builtin_bit_cast(uint16_t, (_Float16)x);
}

// Single-use dense streams bypass cache retention (measured: +5 % on the fused step); the
// in-place p/m/v streams do better with ordinary stores.  The same hint on loads pays for the
// gradient streams that are read exactly once (dense g at the kept positions, compressed gc), not
// for idx or gc16 in the tile kernels (-1.5 %).
__device__ __forceinline__ void store16_stream(void *dst, const uint4 &v)
{
    __builtin_nontemporal_store((u32x4){v.x, v.y, v.z, v.w}, reinterpret_cast<u32x4 *>(dst));
}

__device__ __forceinline__ void store8_stream(void *dst, const uint2 &v)
{
    typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
    __builtin_nontemporal_store((u32x2){v.x, v.y}, reinterpret_cast<u32x2 *>(dst));
}

__device__ __forceinline__ void store_f4_stream(float *dst, const float4 &v)
{
    __builtin_nontemporal_store((f32x4){v.x, v.y, v.z, v.w}, reinterpret_cast<f32x4 *>(dst));
}

__device__ __forceinline__ bool is_nonfinite(float x) { return !(fabsf(x) <= FLT_MAX); }

// One Adam update (Kingma & Ba, Algorithm 1) in fp32.
__device__ __forceinline__ void adam_update(float &p, float &m, float &v, float g, const AdamK &k)
{
    if (k.l2) g = fmaf(k.wd, p, g);
    m = fmaf(k.b1, m, k.omb1 * g);
    v = fmaf(k.b2, v, (k.omb2 * g) * g);
    const float mhat = m * k.rbc1;
    const float denom = sqrtf(v * k.rbc2) + k.eps;
    float upd = mhat / denom;
    if (k.decoupled) upd = fmaf(k.wd, p, upd);
    p = fmaf(-k.lr, upd, p);
}

// One optimizer update; SGD with momentum keeps its single state in m and never touches v.
template <int OPT>
__device__ __forceinline__ void opt_update(float &p, float &m, float &v, float g, const OptK &k)
{
    if (OPT == kOptAdam) {
        adam_update(p, m, v, g, k.adam);
    } else {
        if (k.sgd_wd != 0.f) g = fmaf(k.sgd_wd, p, g);
        m = fmaf(k.sgd_mu, m, g);
        p = fmaf(-k.sgd_lr, m, p);
    }
}

// Clipping coefficient from the device-resident statistics; *skip says the step must do nothing.
__device__ __forceinline__ float guard_coef(const GuardK &gd, bool *skip)
{
    *skip = false;
    float coef = 1.f;
    if (gd.stats) {
        const double ss = gd.stats->sum_squares;
        const int bad = gd.stats->nonfinite;
        if (gd.skip && bad) *skip = true;
        if (gd.max_norm > 0.f) {
            const double c = (double)gd.max_norm / (sqrt(ss) + 1e-6);
            if (c < 1.0) coef = (float)c;
        }
    }
    return coef;
}

__device__ __forceinline__ void pick_work(const LaunchSet &ls, samo_layer *L, int64_t *local)
{
    if (ls.layers) {
        const WgRec r = ls.recs[blockIdx.x];
        *L = ls.layers[r.layer];
        *local = r.local;
    } else {
        *L = ls.one;
        *local = blockIdx.x;
    }
}

// The tile of this workgroup: segments [*s0, *s0 + *nsegs) of *L; *nsegs may be 0 (nothing to do).
__device__ __forceinline__ void pick_tile(const LaunchSet &ls, samo_layer *L, int *s0, int *nsegs)
{
    if (ls.layers) {
        const WgRec r = ls.recs[blockIdx.x];
        *L = ls.layers[r.layer];
        *s0 = (int)(r.local & ((1u << kRecSegShift) - 1u));
        *nsegs = (int)(r.local >> kRecSegShift);
    } else {
        *L = ls.one;
        const int64_t nseg = (ls.one.n + kSeg - 1) / kSeg;
        const int64_t first = (int64_t)blockIdx.x * ls.segs_per_tile;
        *s0 = (int)first;
        *nsegs = (nseg - first < ls.segs_per_tile) ? (int)(nseg - first) : ls.segs_per_tile;
    }
}

// seg_ptr[s] kept inside the compressed arrays: an index that holds more kept elements than the
// arrays have room for (or a table that is no prefix sum) must not carry an access past their end.
__device__ __forceinline__ int slice_bound(const samo_layer &L, int s)
{
    const int64_t c = L.seg_ptr[s];
    return (int)(c < 0 ? 0 : (c > L.nnz ? L.nnz : c));
}

// ------------------------------------------------------------------ tile kernels
// Dense (unpruned) layer: identity index, plain elementwise pass over the tile (one segment, so
// one trip).  A thread takes four consecutive elements — one 16-byte vector of each fp32 array,
// one 8-byte vector of each fp16 array — so every wave-level access is one contiguous run.
template <int MODE, int GSRC, int OPT, int T>
__device__ __forceinline__ void dense_tile(const samo_layer &L, int64_t base, int len, float inv_scale, float coef,
                                           const OptK &k)
{
    const int tid = threadIdx.x;
    float4 *__restrict__ P = reinterpret_cast<float4 *>(L.p + base);
    float4 *__restrict__ M = reinterpret_cast<float4 *>(L.m + base);
    float4 *__restrict__ V = reinterpret_cast<float4 *>(L.v + base);
    // Eight consecutive elements per thread: two 16-byte vectors of each fp32 array, one of each
    // fp16 array (16-byte instead of 8-byte accesses to g and w: 0.72 against 0.70 of peak on the
    // 50304 x 4096 embedding; the gradient, read exactly once, loaded past the caches: 0.74).
    const int nvec8 = len / 8;
    for (int o = tid; o < nvec8; o += T) {
        float p[8], m[8], v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, g[8];
        const float4 pa = P[2 * o], pb = P[2 * o + 1];
        p[0] = pa.x; p[1] = pa.y; p[2] = pa.z; p[3] = pa.w; p[4] = pb.x; p[5] = pb.y; p[6] = pb.z; p[7] = pb.w;
        if (MODE == kModeStep) {
            const float4 ma = M[2 * o], mb = M[2 * o + 1];
            m[0] = ma.x; m[1] = ma.y; m[2] = ma.z; m[3] = ma.w; m[4] = mb.x; m[5] = mb.y; m[6] = mb.z; m[7] = mb.w;
            if (OPT == kOptAdam) {
                const float4 va = V[2 * o], vb = V[2 * o + 1];
                v[0] = va.x; v[1] = va.y; v[2] = va.z; v[3] = va.w; v[4] = vb.x; v[5] = vb.y; v[6] = vb.z; v[7] = vb.w;
            }
            if (GSRC == kGradC32) {
                const f32x4 ga = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(L.gc + base) + 2 * o);
                const f32x4 gb = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(L.gc + base) + 2 * o + 1);
                g[0] = ga.x; g[1] = ga.y; g[2] = ga.z; g[3] = ga.w; g[4] = gb.x; g[5] = gb.y; g[6] = gb.z; g[7] = gb.w;
#pragma unroll
                for (int u = 0; u < 8; ++u) g[u] *= coef;
            } else {
                const u32x4 gq = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>((GSRC == kGradDense ? L.g : L.gc16) + base) + o);
                const uint32_t gw[4] = {gq.x, gq.y, gq.z, gq.w};
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    g[u] = (half_bits_to_float((uint16_t)(gw[u >> 1] >> (16 * (u & 1)))) * inv_scale) * coef;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) opt_update<OPT>(p[u], m[u], v[u], g[u], k);
            P[2 * o] = make_float4(p[0], p[1], p[2], p[3]);
            P[2 * o + 1] = make_float4(p[4], p[5], p[6], p[7]);
            M[2 * o] = make_float4(m[0], m[1], m[2], m[3]);
            M[2 * o + 1] = make_float4(m[4], m[5], m[6], m[7]);
            if (OPT == kOptAdam) {
                V[2 * o] = make_float4(v[0], v[1], v[2], v[3]);
                V[2 * o + 1] = make_float4(v[4], v[5], v[6], v[7]);
            }
        }
        uint32_t wq[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            wq[u] = (uint32_t)float_to_half_bits(p[2 * u]) | ((uint32_t)float_to_half_bits(p[2 * u + 1]) << 16);
        store16_stream(reinterpret_cast<uint4 *>(L.w + base) + o, make_uint4(wq[0], wq[1], wq[2], wq[3]));
    }
    const int nvec = nvec8 * 2;           // elements handled above, in units of four
    for (int e = nvec * 4 + tid; e < len; e += T) {      // ragged end of the layer
        float pe = L.p[base + e];
        if (MODE == kModeStep) {
            float g;
            if (GSRC == kGradC32) g = L.gc[base + e] * coef;
            else g = (half_bits_to_float((GSRC == kGradDense ? L.g : L.gc16)[base + e]) * inv_scale) * coef;
            float me = L.m[base + e], ve = (OPT == kOptAdam) ? L.v[base + e] : 0.f;
            opt_update<OPT>(pe, me, ve, g, k);
            L.p[base + e] = pe;
            L.m[base + e] = me;
            if (OPT == kOptAdam) L.v[base + e] = ve;
        }
        L.w[base + e] = float_to_half_bits(pe);
    }
}

template <int MODE, int GSRC, int OPT, int T>
__device__ __forceinline__ void sparse_tile(const samo_layer &L, int s0, int nsegs, int64_t base, int len,
                                            float inv_scale, float coef, const OptK &k, uint16_t *lds_w)
{
    const int tid = threadIdx.x;
    uint4 *l4 = reinterpret_cast<uint4 *>(lds_w);
    for (int o = tid; o < (len + 7) / 8; o += T) l4[o] = make_uint4(0u, 0u, 0u, 0u);

    const int c0 = slice_bound(L, s0);
    const int c1 = slice_bound(L, s0 + nsegs);
    __syncthreads();

    // The tile's slice [c0, c1) of the compressed arrays is walked in 16-byte vectors of four
    // elements, starting at the vector that holds c0: the in-place fp32 streams move a quarter of
    // the memory instructions of an element-per-lane walk (measured on the flat optimizer kernel:
    // 0.78 against 0.75 of peak; on this kernel with the compressed fp16 gradient 0.75 against 0.73,
    // the expansion at 80 % pruning 0.80 against 0.74).  A vector that straddles c0 or c1 is read
    // whole — its other elements belong to the neighbouring tile and are left alone — and written
    // element by element.  (Used where nothing is gathered from a dense tensor; the step that reads
    // the dense gradient is sparse_tile_dense_grad.)
    const int a0 = c0 & ~3;
    const int nvec = c1 > c0 ? (c1 - a0 + 3) >> 2 : 0;
    const int nnz = (int)L.nnz;
    const int ibase = (int)base;             // a layer's flat size fits int32
    const uint16_t *__restrict__ G = L.g;

    for (int q = tid; q < nvec; q += T) {
        const int e = a0 + 4 * q;            // first element of the vector: a multiple of 4
        int j[4];
        float pp[4], mm[4] = {0.f, 0.f, 0.f, 0.f}, vv[4] = {0.f, 0.f, 0.f, 0.f}, gg[4] = {0.f, 0.f, 0.f, 0.f};
        uint16_t gb[4] = {0, 0, 0, 0};
        bool own[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) own[u] = e + u >= c0 && e + u < c1;
        const bool whole = e + 4 <= nnz;     // the vector lies inside the arrays
        if (whole) {
            const int4 jq = *reinterpret_cast<const int4 *>(L.idx + e);
            const float4 pq = *reinterpret_cast<const float4 *>(L.p + e);
            j[0] = jq.x; j[1] = jq.y; j[2] = jq.z; j[3] = jq.w;
            pp[0] = pq.x; pp[1] = pq.y; pp[2] = pq.z; pp[3] = pq.w;
            if (MODE == kModeStep) {
                const float4 mq = *reinterpret_cast<const float4 *>(L.m + e);
                mm[0] = mq.x; mm[1] = mq.y; mm[2] = mq.z; mm[3] = mq.w;
                if (OPT == kOptAdam) {
                    const float4 vq = *reinterpret_cast<const float4 *>(L.v + e);
                    vv[0] = vq.x; vv[1] = vq.y; vv[2] = vq.z; vv[3] = vq.w;
                }
                if (GSRC == kGradC16) {
                    const uint2 gq = *reinterpret_cast<const uint2 *>(L.gc16 + e);
                    gb[0] = (uint16_t)gq.x; gb[1] = (uint16_t)(gq.x >> 16); gb[2] = (uint16_t)gq.y; gb[3] = (uint16_t)(gq.y >> 16);
                }
                if (GSRC == kGradC32) {
                    const float4 gq = *reinterpret_cast<const float4 *>(L.gc + e);
                    gg[0] = gq.x; gg[1] = gq.y; gg[2] = gq.z; gg[3] = gq.w;
                }
            }
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                j[u] = ibase; pp[u] = 0.f;
                if (own[u]) {
                    j[u] = L.idx[e + u];
                    pp[u] = L.p[e + u];
                    if (MODE == kModeStep) {
                        mm[u] = L.m[e + u];
                        if (OPT == kOptAdam) vv[u] = L.v[e + u];
                        if (GSRC == kGradC16) gb[u] = L.gc16[e + u];
                        if (GSRC == kGradC32) gg[u] = L.gc[e + u];
                    }
                }
            }
        }
        if (MODE == kModeStep && GSRC == kGradDense) {
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (own[u]) gb[u] = __builtin_nontemporal_load(G + j[u]);     // read once: +1 %
        }
        if (MODE == kModeStep) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (own[u]) {
                    const float g = (GSRC == kGradC32) ? gg[u] * coef : (half_bits_to_float(gb[u]) * inv_scale) * coef;
                    opt_update<OPT>(pp[u], mm[u], vv[u], g, k);
                }
            }
            if (whole && own[0] && own[3]) {
                *reinterpret_cast<float4 *>(L.p + e) = make_float4(pp[0], pp[1], pp[2], pp[3]);
                *reinterpret_cast<float4 *>(L.m + e) = make_float4(mm[0], mm[1], mm[2], mm[3]);
                if (OPT == kOptAdam) *reinterpret_cast<float4 *>(L.v + e) = make_float4(vv[0], vv[1], vv[2], vv[3]);
            } else {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (own[u]) {
                        L.p[e + u] = pp[u];
                        L.m[e + u] = mm[u];
                        if (OPT == kOptAdam) L.v[e + u] = vv[u];
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (own[u]) lds_w[j[u] - ibase] = float_to_half_bits(pp[u]);
    }
    __syncthreads();

    uint16_t *__restrict__ W = L.w + base;
    const int nvecw = len / 8;
    for (int o = tid; o < nvecw; o += T) store16_stream(reinterpret_cast<uint4 *>(W) + o, l4[o]);
    for (int e = nvecw * 8 + tid; e < len; e += T) W[e] = lds_w[e];
}

// The step that gathers the dense gradient, with the compressed arrays walked in 16-byte vectors as in
// sparse_tile and the gather done element per lane all the same: a wave passes the positions of its 64
// vectors (256 consecutive compressed elements) through LDS, lane l then reads the gradient at the
// positions of elements l, l + 64, l + 128, l + 192 of that run — consecutive lanes on consecutive kept
// positions, a handful of neighbouring lines per instruction — and the values go back through LDS to
// the lanes that hold the elements' state.  Only the wave's own lanes exchange data: no workgroup barrier.
// Gathering in vector order instead (lane l at elements 4l .. 4l+3) spreads every gather instruction
// over four times as many lines: 0.52 of peak against 0.78; against the element-per-lane walk of
// everything this is level at 90-95 % pruning, 2 % ahead at 80 % and 4 % on the row-clustered 6.7B model.
template <int OPT, int T>
__device__ __forceinline__ void sparse_tile_dense_grad(const samo_layer &L, int s0, int nsegs, int64_t base, int len,
                                                       float inv_scale, float coef, const OptK &k, uint16_t *lds_w,
                                                       int32_t *xj, uint16_t *xg)
{
    const int tid = threadIdx.x, lane = tid & 63;
    uint4 *l4 = reinterpret_cast<uint4 *>(lds_w);
    for (int o = tid; o < (len + 7) / 8; o += T) l4[o] = make_uint4(0u, 0u, 0u, 0u);

    const int c0 = slice_bound(L, s0);
    const int c1 = slice_bound(L, s0 + nsegs);
    __syncthreads();

    const int a0 = c0 & ~3;
    const int nvec = c1 > c0 ? (c1 - a0 + 3) >> 2 : 0;
    const int nnz = (int)L.nnz;
    const int ibase = (int)base;
    const uint16_t *__restrict__ G = L.g;
    int32_t *wj = xj + (tid >> 6) * 256;     // this wave's exchange areas
    uint16_t *wg = xg + (tid >> 6) * 256;

    for (int q0 = 0; q0 < nvec; q0 += T) {   // uniform trip count: every lane takes part in the exchange
        const int q = q0 + tid;
        const int e = a0 + 4 * q;
        int j[4] = {ibase, ibase, ibase, ibase};
        float pp[4] = {0.f, 0.f, 0.f, 0.f}, mm[4] = {0.f, 0.f, 0.f, 0.f}, vv[4] = {0.f, 0.f, 0.f, 0.f};
        bool own[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) own[u] = q < nvec && e + u >= c0 && e + u < c1;
        const bool whole = q < nvec && e + 4 <= nnz;
        if (whole) {
            const int4 jq = *reinterpret_cast<const int4 *>(L.idx + e);
            const float4 pq = *reinterpret_cast<const float4 *>(L.p + e);
            const float4 mq = *reinterpret_cast<const float4 *>(L.m + e);
            j[0] = jq.x; j[1] = jq.y; j[2] = jq.z; j[3] = jq.w;
            pp[0] = pq.x; pp[1] = pq.y; pp[2] = pq.z; pp[3] = pq.w;
            mm[0] = mq.x; mm[1] = mq.y; mm[2] = mq.z; mm[3] = mq.w;
            if (OPT == kOptAdam) {
                const float4 vq = *reinterpret_cast<const float4 *>(L.v + e);
                vv[0] = vq.x; vv[1] = vq.y; vv[2] = vq.z; vv[3] = vq.w;
            }
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (own[u]) {
                    j[u] = L.idx[e + u];
                    pp[u] = L.p[e + u];
                    mm[u] = L.m[e + u];
                    if (OPT == kOptAdam) vv[u] = L.v[e + u];
                }
            }
        }
        // positions to the wave's exchange area in vector order; -1 marks an element that is not this tile's
        *reinterpret_cast<int4 *>(wj + 4 * lane) = make_int4(own[0] ? j[0] : -1, own[1] ? j[1] : -1, own[2] ? j[2] : -1,
                                                             own[3] ? j[3] : -1);
        __builtin_amdgcn_wave_barrier();
        uint16_t got[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int jj = wj[lane + 64 * u];
            got[u] = jj >= 0 ? __builtin_nontemporal_load(G + jj) : (uint16_t)0;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) wg[lane + 64 * u] = got[u];
        __builtin_amdgcn_wave_barrier();
        const uint2 gq = *reinterpret_cast<const uint2 *>(wg + 4 * lane);
        const uint16_t gb[4] = {(uint16_t)gq.x, (uint16_t)(gq.x >> 16), (uint16_t)gq.y, (uint16_t)(gq.y >> 16)};
        __builtin_amdgcn_wave_barrier();     // the areas are free for the next trip
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (own[u]) opt_update<OPT>(pp[u], mm[u], vv[u], (half_bits_to_float(gb[u]) * inv_scale) * coef, k);
        if (whole && own[0] && own[3]) {
            *reinterpret_cast<float4 *>(L.p + e) = make_float4(pp[0], pp[1], pp[2], pp[3]);
            *reinterpret_cast<float4 *>(L.m + e) = make_float4(mm[0], mm[1], mm[2], mm[3]);
            if (OPT == kOptAdam) *reinterpret_cast<float4 *>(L.v + e) = make_float4(vv[0], vv[1], vv[2], vv[3]);
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (own[u]) {
                    L.p[e + u] = pp[u];
                    L.m[e + u] = mm[u];
                    if (OPT == kOptAdam) L.v[e + u] = vv[u];
                }
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (own[u]) lds_w[j[u] - ibase] = float_to_half_bits(pp[u]);
    }
    __syncthreads();

    uint16_t *__restrict__ W = L.w + base;
    const int nvecw = len / 8;
    for (int o = tid; o < nvecw; o += T) store16_stream(reinterpret_cast<uint4 *>(W) + o, l4[o]);
    for (int e = nvecw * 8 + tid; e < len; e += T) W[e] = lds_w[e];
}

template <int MODE, int GSRC, int OPT, int T>
__global__ void __launch_bounds__(T)
tile_kernel(const LaunchSet ls, float inv_scale, const OptK k, const GuardK guard)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_image[];      // ls.max_segs segments of fp16 (and the occupancy padding)
    uint16_t *lds_w = reinterpret_cast<uint16_t *>(lds_image);
    constexpr bool kExchange = MODE == kModeStep && GSRC == kGradDense;
    __shared__ __attribute__((aligned(16))) int32_t xj[kExchange ? T * 4 : 4];      // per wave: 256 positions on their way to the gather
    __shared__ __attribute__((aligned(16))) uint16_t xg[kExchange ? T * 4 : 8];     // and the 256 gradient values on their way back
    bool skip;
    const float coef = guard_coef(guard, &skip);
    if (skip) return;                         // uniform: every workgroup of the launch takes it
    samo_layer L;
    int s0, nsegs;
    pick_tile(ls, &L, &s0, &nsegs);
    if (nsegs > ls.max_segs) nsegs = ls.max_segs;   // a record never holds more; the image must not be overrun whatever it says
    if (nsegs <= 0) return;                   // uniform per workgroup: a record without segments
    const int64_t base = (int64_t)s0 * kSeg;
    const int64_t rest = L.n - base;
    const int len = rest < (int64_t)nsegs * kSeg ? (int)rest : nsegs * kSeg;
    if (L.seg_ptr == nullptr)                 // dense (unpruned) layer
        dense_tile<MODE, GSRC, OPT, T>(L, base, len, inv_scale, coef, k);
    else if (kExchange)
        sparse_tile_dense_grad<OPT, T>(L, s0, nsegs, base, len, inv_scale, coef, k, lds_w, xj, xg);
    else
        sparse_tile<MODE, GSRC, OPT, T>(L, s0, nsegs, base, len, inv_scale, coef, k, lds_w);
}

// ------------------------------------------------------------------ single-precision tile kernel
// The same tile scheme with theta32 as the dense side: the kept values of the tile are read from
// the dense fp32 parameters themselves, stepped, and dropped into a zero-filled fp32 image of the
// tile in LDS, which leaves as whole 16-byte non-temporal stores — pruned positions come out +0,
// the optimizer state m, v is the only compressed fp32 traffic.
template <int T>
__device__ __forceinline__ void dense_tile_fp32(const samo_layer &L, int64_t base, int len, float factor, float coef,
                                                const OptK &k)
{
    const int tid = threadIdx.x;
    float4 *__restrict__ W = reinterpret_cast<float4 *>(L.w32 + base);
    float4 *__restrict__ M = reinterpret_cast<float4 *>(L.m + base);
    float4 *__restrict__ V = reinterpret_cast<float4 *>(L.v + base);
    const f32x4 *__restrict__ G = reinterpret_cast<const f32x4 *>(L.g32 + base);
    const int nvec = len / 4;
    for (int o = tid; o < nvec; o += T) {
        float4 p = W[o], m = M[o], v = V[o];
        const f32x4 g = __builtin_nontemporal_load(G + o);
        adam_update(p.x, m.x, v.x, (g.x * factor) * coef, k.adam);
        adam_update(p.y, m.y, v.y, (g.y * factor) * coef, k.adam);
        adam_update(p.z, m.z, v.z, (g.z * factor) * coef, k.adam);
        adam_update(p.w, m.w, v.w, (g.w * factor) * coef, k.adam);
        W[o] = p;
        M[o] = m;
        V[o] = v;
    }
    for (int e = nvec * 4 + tid; e < len; e += T) {                  // ragged end of the layer
        float pe = L.w32[base + e], me = L.m[base + e], ve = L.v[base + e];
        adam_update(pe, me, ve, (L.g32[base + e] * factor) * coef, k.adam);
        L.w32[base + e] = pe;
        L.m[base + e] = me;
        L.v[base + e] = ve;
    }
}

template <int T>
__device__ __forceinline__ void sparse_tile_fp32(const samo_layer &L, int s0, int nsegs, int64_t base, int len,
                                                 float factor, float coef, const OptK &k, float *lds_f)
{
    const int tid = threadIdx.x;
    float4 *l4 = reinterpret_cast<float4 *>(lds_f);
    for (int o = tid; o < (len + 3) / 4; o += T) l4[o] = make_float4(0.f, 0.f, 0.f, 0.f);
    const int c0 = slice_bound(L, s0);
    const int c1 = slice_bound(L, s0 + nsegs);
    __syncthreads();

    const int cnt = c1 > c0 ? c1 - c0 : 0;
    const int32_t *__restrict__ IDX = L.idx + c0;
    float *__restrict__ M = L.m + c0;
    float *__restrict__ V = L.v + c0;
    const float *__restrict__ G = L.g32;
    const float *W = L.w32;                  // read at the kept positions here, rewritten as a whole tile below
    const int ibase = (int)base;

    constexpr int U = kTileUnrollFp32;
    for (int r0 = tid; r0 < cnt; r0 += U * T) {
        int j[U];
        float pp[U], mm[U], vv[U], gg[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int r = r0 + u * T;
            j[u] = ibase; pp[u] = 0.f; mm[u] = 0.f; vv[u] = 0.f; gg[u] = 0.f;
            if (r < cnt) {
                j[u] = IDX[r];
                mm[u] = M[r];
                vv[u] = V[r];
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (r0 + u * T < cnt) {
                gg[u] = __builtin_nontemporal_load(G + j[u]);
                pp[u] = W[j[u]];
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int r = r0 + u * T;
            if (r < cnt) {
                adam_update(pp[u], mm[u], vv[u], (gg[u] * factor) * coef, k.adam);
                M[r] = mm[u];
                V[r] = vv[u];
                lds_f[j[u] - ibase] = pp[u];
            }
        }
    }
    __syncthreads();                          // every read of this tile of w32 has happened

    float *Wout = L.w32 + base;              // aliases W: no restrict
    const int nvec = len / 4;
    for (int o = tid; o < nvec; o += T) store_f4_stream(Wout + 4 * o, l4[o]);
    for (int e = nvec * 4 + tid; e < len; e += T) Wout[e] = lds_f[e];
}

template <int T>
__global__ void __launch_bounds__(T)
tile_fp32_kernel(const LaunchSet ls, float factor, const OptK k, const GuardK guard)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_image[];      // ls.max_segs segments of fp32 (and the occupancy padding)
    float *lds_f = reinterpret_cast<float *>(lds_image);
    bool skip;
    const float coef = guard_coef(guard, &skip);
    if (skip) return;
    samo_layer L;
    int s0, nsegs;
    pick_tile(ls, &L, &s0, &nsegs);
    if (nsegs > ls.max_segs) nsegs = ls.max_segs;
    if (nsegs <= 0) return;
    const int64_t base = (int64_t)s0 * kSeg;
    const int64_t rest = L.n - base;
    const int len = rest < (int64_t)nsegs * kSeg ? (int)rest : nsegs * kSeg;
    if (L.seg_ptr == nullptr)
        dense_tile_fp32<T>(L, base, len, factor, coef, k);
    else
        sparse_tile_fp32<T>(L, s0, nsegs, base, len, factor, coef, k, lds_f);
}

// ------------------------------------------------------------------ statistics helpers
// Sum over the 64 lanes of a wave, the same value returned to every lane.  Data-parallel
// primitives move the operands between lanes inside the vector ALU (row shifts within 16 lanes,
// then two row broadcasts), which is a handful of cycles per step where a shuffle through the LDS
// crossbar costs a round trip; the order of the additions is fixed.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_add_f64(double x)
{
    const int lo = __double2loint(x), hi = __double2hiint(x);
    // lanes the pattern does not feed read 0.0 (bound_ctrl), rows outside ROW_MASK keep x + 0.0
    const int lo2 = __builtin_amdgcn_update_dpp(0, lo, CTRL, ROW_MASK, 0xf, true);
    const int hi2 = __builtin_amdgcn_update_dpp(0, hi, CTRL, ROW_MASK, 0xf, true);
    return x + __hiloint2double(hi2, lo2);
}

__device__ __forceinline__ double wave_sum_f64(double x)
{
    x = dpp_add_f64<0x111, 0xf>(x);           // row_shr:1  (inclusive scan within each row of 16 lanes)
    x = dpp_add_f64<0x112, 0xf>(x);           // row_shr:2
    x = dpp_add_f64<0x114, 0xf>(x);           // row_shr:4
    x = dpp_add_f64<0x118, 0xf>(x);           // row_shr:8
    x = dpp_add_f64<0x142, 0xa>(x);           // row_bcast:15 into rows 1 and 3
    x = dpp_add_f64<0x143, 0xc>(x);           // row_bcast:31 into rows 2 and 3: lane 63 holds the total
    const int lo = __builtin_amdgcn_readlane(__double2loint(x), 63);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(x), 63);
    return __hiloint2double(hi, lo);
}

// A flat workgroup is one wave: its (sum of squares, flag) partial is a wave reduction, fixed
// order, deterministic.  Consecutive workgroups run on different XCDs (round-robin), each with its
// own L2; the slot permutation gives every XCD a contiguous run of the partials array, so the
// 16-byte stores of one XCD fill whole cache lines in its L2 instead of eight L2s each holding an
// eighth of every line.
static_assert(kFlatThreads == 64, "write_partial assumes one wave per flat workgroup");
// Whether slot s of a launch of `grid` workgroups was written (the last few may belong to
// workgroups beyond the grid).
__device__ __forceinline__ bool partial_slot_used(int64_t s, unsigned grid)
{
    const unsigned per_xcd = (grid + 7u) / 8u;
    const unsigned block = (unsigned)(s % per_xcd) * 8u + (unsigned)(s / per_xcd);
    return block < grid;
}

__device__ __forceinline__ void write_partial(double ss, int bad, StatPartial *__restrict__ partials)
{
    ss = wave_sum_f64(ss);
    bad = __any(bad) ? 1 : 0;
    if (threadIdx.x == 0) {
        const unsigned per_xcd = (gridDim.x + 7u) / 8u;
        const unsigned slot = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
        partials[slot].sum_squares = ss;
        partials[slot].nonfinite = bad;
    }
}

// ------------------------------------------------------------------ flat kernels over the compressed arrays
// Gradient compression.  SRC: where a value comes from (dense g at idx, gc16, gc); OUT: what is
// written (fp32 unscaled gc, fp16 gc16 with optional accumulation, nothing).  When `partials` is
// given, the sum of squares and the non-finite flag of the unscaled values are reduced as well.
// One workgroup (a single wave) per chunk record; with statistics it leaves one partial, which
// stats_reduce_kernel / stats_finalize_kernel sum afterwards (a grid of padded slots: see
// launch_gather).
template <int OUT>
__global__ void __launch_bounds__(kFlatThreads)
gather_kernel(const LaunchSet ls, int src, float inv_scale, int accumulate, StatPartial *__restrict__ partials)
{
    double ss = 0.0;
    int bad = 0;
    static_assert(kChunk == 4 * kFlatThreads, "one float4 per thread and chunk record");
    samo_layer L;
    int64_t chunk;
    pick_work(ls, &L, &chunk);
    const int64_t nnz = L.nnz;
    const bool identity = (L.idx == nullptr);             // dense layer: position i is element i
    const int64_t i = chunk * kChunk + (int64_t)threadIdx.x * 4;
    const int cnt = (nnz - i >= 4) ? 4 : (nnz - i > 0 ? (int)(nnz - i) : 0);
    uint16_t hb[4] = {0, 0, 0, 0};
    float fv[4] = {0.f, 0.f, 0.f, 0.f};
    if (src == kGradC32 || (src == kGradDense32 && identity)) {
        const float *S = (src == kGradC32) ? L.gc : L.g32;
        if (cnt == 4) {
            const float4 q = *reinterpret_cast<const float4 *>(S + i);
            fv[0] = q.x; fv[1] = q.y; fv[2] = q.z; fv[3] = q.w;
        } else {
            for (int e = 0; e < cnt; ++e) fv[e] = S[i + e];
        }
    } else if (src == kGradC16 || identity) {
        const uint16_t *S = (src == kGradC16) ? L.gc16 : L.g;
        if (cnt == 4) {
            const uint2 q = *reinterpret_cast<const uint2 *>(S + i);
            hb[0] = (uint16_t)q.x; hb[1] = (uint16_t)(q.x >> 16); hb[2] = (uint16_t)q.y; hb[3] = (uint16_t)(q.y >> 16);
        } else {
            for (int e = 0; e < cnt; ++e) hb[e] = S[i + e];
        }
    } else {
        // A dense gradient read at the kept positions.  The lane's four positions come as one 16-byte
        // vector, but the gather is done element per lane: the wave passes its 256 positions through
        // LDS, lane l reads the gradient at those of elements l, l + 64, l + 128, l + 192 — consecutive
        // lanes on consecutive kept positions, a handful of neighbouring lines per instruction — and the
        // values come back through LDS in vector order.  One wave per workgroup: no barrier needed.
        __shared__ __attribute__((aligned(16))) int32_t xj[kChunk];
        __shared__ __attribute__((aligned(16))) uint32_t xv[kChunk];
        int j4[4] = {-1, -1, -1, -1};                                // -1: beyond the layer's last kept element
        if (cnt == 4) {
            int4 j;
            if (OUT == kOutF32) {                                // measured: +2 % here, -1.5 % with fp16 output
                const i32x4 jq = __builtin_nontemporal_load(reinterpret_cast<const i32x4 *>(L.idx + i));
                j = make_int4(jq.x, jq.y, jq.z, jq.w);
            } else {
                j = *reinterpret_cast<const int4 *>(L.idx + i);
            }
            j4[0] = j.x; j4[1] = j.y; j4[2] = j.z; j4[3] = j.w;
        } else {
            for (int e = 0; e < cnt; ++e) j4[e] = L.idx[i + e];
        }
        const int lane = threadIdx.x;
        *reinterpret_cast<int4 *>(xj + 4 * lane) = make_int4(j4[0], j4[1], j4[2], j4[3]);
        __builtin_amdgcn_wave_barrier();
        uint32_t got[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int jj = xj[lane + 64 * u];
            if (src == kGradDense32) got[u] = jj >= 0 ? __float_as_uint(L.g32[jj]) : 0u;
            else got[u] = jj >= 0 ? (uint32_t)L.g[jj] : 0u;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) xv[lane + 64 * u] = got[u];
        __builtin_amdgcn_wave_barrier();
        const uint4 back = *reinterpret_cast<const uint4 *>(xv + 4 * lane);
        if (src == kGradDense32) {
            fv[0] = __uint_as_float(back.x); fv[1] = __uint_as_float(back.y); fv[2] = __uint_as_float(back.z); fv[3] = __uint_as_float(back.w);
        } else {
            hb[0] = (uint16_t)back.x; hb[1] = (uint16_t)back.y; hb[2] = (uint16_t)back.z; hb[3] = (uint16_t)back.w;
        }
    }
    if (OUT == kOutF16) {
        if (accumulate) {                                  // one correctly rounded half addition
            uint16_t old[4] = {0, 0, 0, 0};
            if (cnt == 4) {
                const uint2 q = *reinterpret_cast<const uint2 *>(L.gc16 + i);
                old[0] = (uint16_t)q.x; old[1] = (uint16_t)(q.x >> 16); old[2] = (uint16_t)q.y; old[3] = (uint16_t)(q.y >> 16);
            } else {
                for (int e = 0; e < cnt; ++e) old[e] = L.gc16[i + e];
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const _Float16 sum = __builtin_bit_cast(_Float16, old[e]) + __builtin_bit_cast(_Float16, hb[e]);
                hb[e] = __builtin_bit_cast(uint16_t, sum);
            }
        }
        if (cnt == 4) {
            store8_stream(L.gc16 + i, make_uint2((uint32_t)hb[0] | ((uint32_t)hb[1] << 16),
                                                 (uint32_t)hb[2] | ((uint32_t)hb[3] << 16)));   // +4 % over a plain store
        } else {
            for (int e = 0; e < cnt; ++e) L.gc16[i + e] = hb[e];
        }
    }
    if (src != kGradC32 && src != kGradDense32) {
#pragma unroll
        for (int e = 0; e < 4; ++e) fv[e] = half_bits_to_float(hb[e]) * inv_scale;
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) fv[e] = fv[e] * inv_scale;
    }
    if (OUT == kOutF32) {
        if (cnt == 4) store_f4_stream(L.gc + i, make_float4(fv[0], fv[1], fv[2], fv[3]));
        else for (int e = 0; e < cnt; ++e) L.gc[i + e] = fv[e];
    }
    if (partials) {
        for (int e = 0; e < cnt; ++e) {
            ss += (double)fv[e] * (double)fv[e];
            bad |= is_nonfinite(fv[e]) ? 1 : 0;
        }
    }
    if (partials) write_partial(ss, bad, partials);
}

// Statistics of a compressed gradient (gc16 or gc) with nothing written: no gather and no store
// to hide, so one record per wave would leave the launch bound by its own overhead (512 bytes read
// per wave).  Here a wave takes kStatRun chunk records, kStatAhead at a time with their loads in
// flight together, and still leaves one partial per record, each reduced as gather_kernel reduces
// it and stored in the slot gather_kernel would use: the sums that follow, and so the bits of the
// result, are those of every other way to the same statistics.  The records of a wave are the ones
// whose slots are consecutive (every eighth record), so lane k stores partial k and the wave
// writes one run of kStatRun partials.  The loads of a group sit in straight-line code (descriptors read
// unconditionally at a clamped record, the 4-element vector under a lane predicate); the ragged
// end of a layer, at most one lane of one record, is read element by element afterwards.
constexpr int kStatRun = 8;
constexpr int kStatAhead = 8;        // records whose loads are in flight together

template <int SRC>
__global__ void __launch_bounds__(kFlatThreads)
stats_compressed_kernel(const LaunchSet ls, float inv_scale, StatPartial *__restrict__ partials)
{
    static_assert(SRC == kGradC16 || SRC == kGradC32, "compressed sources only");
    static_assert(kStatRun <= kFlatThreads && kStatRun % kStatAhead == 0, "lane k keeps partial k");
    constexpr int kWords = (SRC == kGradC32) ? 4 : 2;     // 32-bit words of a lane's four elements
    const unsigned total = (unsigned)ls.wgs;              // records, and workgroups of the launch this one stands for
    const unsigned per_xcd = (total + 7u) / 8u;
    const unsigned run = blockIdx.x & 7u;                 // which eighth of the slots
    const unsigned base = (blockIdx.x >> 3) * kStatRun;   // first slot of the wave within that eighth
    double mine_ss = 0.0;
    int mine_bad = 0;
    bool have = false;
    typedef const __attribute__((address_space(1))) uint32_t *GlobalWords;     // the arrays live in device memory
    typedef const __attribute__((address_space(1))) uint16_t *GlobalHalves;
    typedef unsigned int Words2 __attribute__((ext_vector_type(2)));
    typedef const __attribute__((address_space(1))) Words2 *GlobalWords2;
    typedef const __attribute__((address_space(1))) u32x4 *GlobalWords4;
    for (int r0 = 0; r0 < kStatRun; r0 += kStatAhead) {
        uint32_t q[kStatAhead][kWords];
        GlobalWords at[kStatAhead];                        // the lane's first element
        int cnt[kStatAhead];
        bool live[kStatAhead];
        WgRec r[kStatAhead];
        int64_t nnz[kStatAhead];
        const void *arr[kStatAhead];
#pragma unroll
        for (int u = 0; u < kStatAhead; ++u) {
            const unsigned rec = run + 8u * (base + r0 + u);
            live[u] = (base + r0 + u) < per_xcd && rec < total;
            r[u] = ls.recs[live[u] ? rec : 0u];
        }
#pragma unroll
        for (int u = 0; u < kStatAhead; ++u) {
            const samo_layer *L = ls.layers + r[u].layer;
            nnz[u] = L->nnz;
            arr[u] = (SRC == kGradC32) ? (const void *)L->gc : (const void *)L->gc16;
        }
#pragma unroll
        for (int u = 0; u < kStatAhead; ++u) {
            // a record beyond the launch counts as one beyond its layer's end: nothing to read
            const int64_t i = live[u] ? r[u].local * kChunk + (int64_t)threadIdx.x * 4 : INT64_MAX / 2;
            cnt[u] = (nnz[u] - i >= 4) ? 4 : (nnz[u] - i > 0 ? (int)(nnz[u] - i) : 0);
            const int64_t off = live[u] ? i : 0;
            at[u] = (SRC == kGradC32) ? (GlobalWords)((const float *)arr[u] + off)
                                      : (GlobalWords)((const uint16_t *)arr[u] + off);
#pragma unroll
            for (int w = 0; w < kWords; ++w) q[u][w] = 0u;
            if (cnt[u] == 4) {
                if (SRC == kGradC32) {
                    const u32x4 x = *(GlobalWords4)at[u];
                    q[u][0] = x.x; q[u][1] = x.y; q[u][kWords - 2] = x.z; q[u][kWords - 1] = x.w;
                } else {
                    const Words2 x = *(GlobalWords2)at[u];
                    q[u][0] = x.x; q[u][1] = x.y;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kStatAhead; ++u) {
            if (cnt[u] > 0 && cnt[u] < 4) {
#pragma unroll
                for (int e = 0; e < 3; ++e) {
                    if (e >= cnt[u]) continue;
                    if (SRC == kGradC32) q[u][e] = at[u][e];
                    else q[u][e >> 1] |= (uint32_t)((GlobalHalves)at[u])[e] << (16 * (e & 1));
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kStatAhead; ++u) {
            double ss = 0.0;
            int bad = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float raw = (SRC == kGradC32) ? __uint_as_float(q[u][e])
                                                    : half_bits_to_float((uint16_t)(q[u][e >> 1] >> (16 * (e & 1))));
                if (e < cnt[u]) {
                    const float x = raw * inv_scale;
                    ss += (double)x * (double)x;
                    bad |= is_nonfinite(x) ? 1 : 0;
                }
            }
            ss = wave_sum_f64(ss);
            bad = __any(bad) ? 1 : 0;
            if ((int)threadIdx.x == r0 + u) { mine_ss = ss; mine_bad = bad; have = live[u]; }
        }
    }
    if (have) {
        const unsigned slot = run * per_xcd + base + threadIdx.x;
        partials[slot].sum_squares = mine_ss;
        partials[slot].nonfinite = mine_bad;
    }
}

// First level of the reduction: workgroup b sums the contiguous slice [b * per, (b + 1) * per) of
// the partials into out[b]; thread t of it takes elements t, t + 256, ... of the slice, then a
// fixed tree.  Every order is fixed by (count, per) alone.
constexpr int kReduceThreads = 256;

__global__ void __launch_bounds__(kReduceThreads)
stats_reduce_kernel(const StatPartial *__restrict__ partials, int64_t count, unsigned gather_grid, int64_t per,
                    StatPartial *__restrict__ out)
{
    __shared__ double sh_ss[kReduceThreads / 64];
    __shared__ int sh_bad[kReduceThreads / 64];
    const int64_t lo = (int64_t)blockIdx.x * per;
    const int64_t hi = (lo + per < count) ? lo + per : count;
    double ss = 0.0;
    int bad = 0;
    constexpr int kAhead = 4;                 // loads in flight per thread; the additions keep their order
    for (int64_t i0 = lo + threadIdx.x; i0 < hi; i0 += (int64_t)kAhead * kReduceThreads) {
        StatPartial part[kAhead];
#pragma unroll
        for (int a = 0; a < kAhead; ++a) {
            const int64_t i = i0 + (int64_t)a * kReduceThreads;
            part[a].sum_squares = 0.0;
            part[a].nonfinite = 0;
            if (i < hi && partial_slot_used(i, gather_grid)) part[a] = partials[i];
        }
#pragma unroll
        for (int a = 0; a < kAhead; ++a) {
            ss += part[a].sum_squares;
            bad |= part[a].nonfinite != 0;
        }
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    ss = wave_sum_f64(ss);
    bad = __any(bad) ? 1 : 0;
    if (lane == 0) { sh_ss[wave] = ss; sh_bad[wave] = bad; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        int b = 0;
        for (int w = 0; w < kReduceThreads / 64; ++w) { t += sh_ss[w]; b |= sh_bad[w]; }
        out[blockIdx.x].sum_squares = t;
        out[blockIdx.x].nonfinite = b;
    }
}

// Last level: sums up to a few thousand partials in a fixed order: thread t takes partials
// t, t + 1024, ..., then one fixed-shape tree over the 1024 threads.
constexpr int kFinalizeThreads = 1024;

__global__ void __launch_bounds__(kFinalizeThreads)
stats_finalize_kernel(const StatPartial *__restrict__ partials, int64_t count, unsigned gather_grid,
                      samo_grad_stats *__restrict__ out)
{
    __shared__ double sh_ss[kFinalizeThreads / 64];
    __shared__ int sh_bad[kFinalizeThreads / 64];
    double ss = 0.0;
    int bad = 0;
    constexpr int kAhead = 8;                 // loads in flight per thread; the additions keep their order
    for (int64_t i0 = threadIdx.x; i0 < count; i0 += (int64_t)kAhead * kFinalizeThreads) {
        StatPartial part[kAhead];
#pragma unroll
        for (int a = 0; a < kAhead; ++a) {
            const int64_t i = i0 + (int64_t)a * kFinalizeThreads;
            part[a].sum_squares = 0.0;
            part[a].nonfinite = 0;
            // gather_grid != 0: the partials come straight from a gather launch of that many workgroups
            if (i < count && (gather_grid == 0 || partial_slot_used(i, gather_grid))) part[a] = partials[i];
        }
#pragma unroll
        for (int a = 0; a < kAhead; ++a) {
            ss += part[a].sum_squares;
            bad |= part[a].nonfinite != 0;
        }
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    ss = wave_sum_f64(ss);
    bad = __any(bad) ? 1 : 0;
    if (lane == 0) { sh_ss[wave] = ss; sh_bad[wave] = bad; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        int b = 0;
        for (int w = 0; w < kFinalizeThreads / 64; ++w) { t += sh_ss[w]; b |= sh_bad[w]; }
        out->sum_squares = t;
        out->nonfinite = b;
        out->reserved = 0;
    }
}

// Optimizer step over the compressed arrays with an fp32 compressed gradient.
template <int OPT>
__global__ void __launch_bounds__(kFlatThreads)
flat_step_kernel(const LaunchSet ls, const OptK k, const GuardK guard)
{
    bool skip;
    const float coef = guard_coef(guard, &skip);
    if (skip) return;
    samo_layer L;
    int64_t chunk;
    pick_work(ls, &L, &chunk);
    const int64_t nnz = L.nnz;
    float *__restrict__ P = L.p;
    float *__restrict__ M = L.m;
    float *__restrict__ V = L.v;
    const float *__restrict__ GC = L.gc;
#pragma unroll
    for (int it = 0; it < kChunk / (4 * kFlatThreads); ++it) {
        const int64_t i = chunk * kChunk + ((int64_t)it * kFlatThreads + threadIdx.x) * 4;
        if (i + 4 <= nnz) {
            float4 p = *reinterpret_cast<const float4 *>(P + i);
            float4 m = *reinterpret_cast<const float4 *>(M + i);
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (OPT == kOptAdam) v = *reinterpret_cast<const float4 *>(V + i);
            const f32x4 gq = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(GC + i));   // read once: +2 %
            const float4 g = make_float4(gq.x, gq.y, gq.z, gq.w);
            opt_update<OPT>(p.x, m.x, v.x, g.x * coef, k);
            opt_update<OPT>(p.y, m.y, v.y, g.y * coef, k);
            opt_update<OPT>(p.z, m.z, v.z, g.z * coef, k);
            opt_update<OPT>(p.w, m.w, v.w, g.w * coef, k);
            *reinterpret_cast<float4 *>(P + i) = p;
            *reinterpret_cast<float4 *>(M + i) = m;
            if (OPT == kOptAdam) *reinterpret_cast<float4 *>(V + i) = v;
        } else {
            for (int64_t e = i; e < nnz; ++e) {
                float p = P[e], m = M[e], v = (OPT == kOptAdam) ? V[e] : 0.f;
                opt_update<OPT>(p, m, v, GC[e] * coef, k);
                P[e] = p;
                M[e] = m;
                if (OPT == kOptAdam) V[e] = v;
            }
        }
    }
}

// ------------------------------------------------------------------ tile records of a plan
// Record k of a pruned layer owns the segments s whose running weight C(s) = kSegCost * s +
// kNnzCost * seg_ptr[s] (the weight of everything before s) falls in
// [k * tile_cost, (k + 1) * tile_cost): C is increasing, so the records partition the layer, each
// weighs about tile_cost, and none holds more than tile_cost_segs(tile_cost) segments.  seg_ptr is the prefix
// sum already, so a record's bounds are two binary searches, independent of every other record.
// A record can be empty (a single segment heavier than tile_cost spans two buckets).  An unpruned
// layer gets one record per segment.
__device__ __forceinline__ int64_t first_seg_with_cost(const int32_t *__restrict__ seg_ptr, int64_t nseg, int64_t target)
{
    int64_t lo = 0, hi = nseg;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        const int64_t cost = kSegCost * mid + kNnzCost * (int64_t)seg_ptr[mid];
        if (cost < target) lo = mid + 1; else hi = mid;
    }
    return lo;
}

__global__ void __launch_bounds__(kThreads)
build_tile_recs_kernel(const samo_layer *__restrict__ layers, const int64_t *__restrict__ rec_start, int num_layers,
                       int64_t total, int64_t tile_cost, int max_segs, WgRec *__restrict__ recs)
{
    const int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (t >= total) return;
    int lo = 0, hi = num_layers;                // the last layer whose first record is <= t
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (rec_start[mid] <= t) lo = mid; else hi = mid;
    }
    const samo_layer L = layers[lo];
    const int64_t k = t - rec_start[lo];
    const int64_t nrec = rec_start[lo + 1] - rec_start[lo];
    const int64_t nseg = (L.n + kSeg - 1) / kSeg;
    int64_t first = k, count = 1;
    if (L.seg_ptr != nullptr) {
        first = (k == 0) ? 0 : first_seg_with_cost(L.seg_ptr, nseg, k * tile_cost);
        const int64_t end = (k + 1 == nrec) ? nseg : first_seg_with_cost(L.seg_ptr, nseg, (k + 1) * tile_cost);
        count = end - first;
        if (count < 0) count = 0;                       // only with a seg_ptr that is not a prefix sum:
        if (count > max_segs) count = max_segs;         // stay inside the workgroup's LDS image
    }
    recs[t].layer = lo;
    recs[t].local = (uint32_t)first | ((uint32_t)count << kRecSegShift);
}

// Chunk records of the flat kernels: record t is chunk t - rec_start[l] of the layer l that holds it.
__global__ void __launch_bounds__(kThreads)
build_chunk_recs_kernel(const int64_t *__restrict__ rec_start, int num_layers, int64_t total, WgRec *__restrict__ recs)
{
    const int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (t >= total) return;
    int lo = 0, hi = num_layers;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (rec_start[mid] <= t) lo = mid; else hi = mid;
    }
    recs[t].layer = lo;
    recs[t].local = (uint32_t)(t - rec_start[lo]);
}

// The plan's layer table: descriptors and record starts arrive in the kernel arguments and are
// written to the caller's workspace.  nnz of a pruned layer becomes what its index holds now — the
// last entry of seg_ptr — capped by the capacity the host gave.
__global__ void __launch_bounds__(64)
plan_write_kernel(const PlanBatch batch, const PlanTables t)
{
    const int k = threadIdx.x;
    if (k < batch.count) {
        samo_layer L = batch.layer[k];
        if (L.seg_ptr != nullptr) {
            const int64_t nseg = (L.n + kSeg - 1) / kSeg;
            const int64_t have = L.seg_ptr[nseg];
            L.nnz = have < 0 ? 0 : (have < L.nnz ? have : L.nnz);
        }
        t.layers[batch.first + k] = L;
    }
    if (k <= batch.count) {
        t.tile_start[batch.first + k] = batch.tile_start[k];
        t.chunk_start[batch.first + k] = batch.chunk_start[k];
    }
}

// ------------------------------------------------------------------ diagnostic copy
// 16 bytes per thread, 4 KiB per workgroup: the fastest plain-copy shape measured on MI355X.
__global__ void __launch_bounds__(kThreads)
copy_kernel(uint4 *__restrict__ dst, const uint4 *__restrict__ src, int64_t nvec)
{
    const int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (o < nvec) dst[o] = src[o];
}

}  // namespace

// Occupancy targets.  MI355X streams fastest with a bounded amount of traffic in flight per
// compute unit; one workgroup too many per CU and bandwidth drops by 5-15 % (measured: the fused
// step at 90 % sparsity reaches 6.2 TB/s with 6 workgroups per CU, 5.5 with 7).  Tile workgroups
// all move about kTileCost bytes, so one target serves every density; it is enforced by padding
// the LDS request: a workgroup that asks for a size between LDS/(target+1) and LDS/target fits
// exactly `target` times.  samo_debug_set overrides the targets (tuning aid; 0 = no cap).
constexpr int kLdsPerCu = 160 * 1024;
static int lds_pad_for(int target_wgs, int static_bytes)
{
    if (target_wgs <= 0) return 0;
    const int want = (kLdsPerCu / (target_wgs + 1) + kLdsPerCu / target_wgs) / 2;
    return want > static_bytes ? want - static_bytes : 0;
}
// Dynamic LDS of a tile launch: the image of the largest tile, or more where the occupancy target asks for it.
static int tile_lds_request(int target_wgs, int static_bytes, int image_bytes)
{
    const int pad = lds_pad_for(target_wgs, static_bytes);
    return pad > image_bytes ? pad : image_bytes;
}

static int occ_tile_step(int gsrc, int opt, float keep)
{
    // a step that reads the dense gradient keeps whole dense lines in flight: 6 workgroups per CU;
    // with a compressed gradient (half the bytes per workgroup) every wave slot is worth filling at
    // 90 % pruning and above (8 workgroups: 0.75 of peak against 0.72 with 6), while at 80 % the
    // in-place streams are over half the traffic and 6 is the optimum again (0.74 against 0.68 with 8)
    // (where the model keeps so little that its tiles have twice the weight: 4, and 6 with the compressed gradient)
    const bool sparse = keep < (float)kSparseKeep;
    if (gsrc == kGradDense) return knob(SAMO_KNOB_OCC_TILE_STEP, sparse ? (opt == kOptSgd ? 3 : 4) : 6);
    return knob(SAMO_KNOB_OCC_TILE_C16, (sparse || keep > 0.15f) ? 6 : 0);
}

static int occ_tile_decompress(float keep)
{
    return knob(SAMO_KNOB_OCC_TILE_DECOMP, keep < (float)kSparseKeep ? 8 : 0);
}

// Flat gather: one wave holds 1 KiB of indices and about 512 / keep bytes of dense lines in
// flight; aim at ~75 KiB per CU.
static int occ_flat_gather(int out, int src, float keep, bool with_stats)
{
    const int forced = knob(SAMO_KNOB_OCC_FLAT_GATHER, -1);
    const int forced_stats = knob(SAMO_KNOB_OCC_FLAT_STATS, -1);
    if (with_stats && forced_stats >= 0) return forced_stats;
    if (!with_stats && forced >= 0) return forced;
    if (src != kGradDense && src != kGradDense32) return with_stats ? 20 : 12;
    // Waves per compute unit.  A wave's share of the dense gradient grows as the kept fraction
    // falls, and with it the lines a wave has in flight; the measured optima on the GPT-3 2.7B
    // masks are narrow (10 at 5 % kept, 14-15 at 10 %, 22-24 at 20 %: two waves off cost 5-8 %).
    float t = 5.7f + 87.f * keep;
    if (t < 10.f) t = 10.f;
    // the statistics add an arithmetic tail during which a wave has no memory traffic in flight:
    // more waves have to be resident for the same traffic in flight, most when the wave also
    // has a store to retire (optima: 15 / 24 / 28 with the fp16 store, 11 / 16 / 27 without; 24 on the row-clustered 6.7B model, whose
    // dense embedding lifts its kept fraction to 0.13)
    if (with_stats) t *= (out == kOutNone) ? 1.3f : 1.4f;
    return t > 30.f ? 0 : (int)(t + 0.5f);
}

static int occ_flat_step()
{
    return knob(SAMO_KNOB_OCC_FLAT_STEP, 13);     // a narrow optimum: 12-15 waves per CU by size of the arrays, 16 loses 7 %
}

#define SAMO_LAUNCH_TILE(M, G, O)                                                                          \
    tile_kernel<M, G, O, kTileThreads><<<dim3((unsigned)ls.wgs), dim3(kTileThreads), pad, s>>>(ls, inv_scale, k, guard)

hipError_t launch_tile(int mode, int gsrc, int opt, const LaunchSet &ls, float inv_scale, const OptK &k,
                       const GuardK &guard, hipStream_t s)
{
    if (ls.wgs <= 0) return hipSuccess;
    if (ls.max_segs < 1 || ls.max_segs > kMaxTileSegs) return hipErrorInvalidValue;
    // static LDS of the kernel: for the step that gathers the dense gradient the waves' exchange areas;
    // dynamic: the tile's fp16 image
    const int static_lds = mode == kModeStep && gsrc == kGradDense ? kTileThreads * 4 * 6 : 32;
    const int pad = tile_lds_request(mode == kModeDecompress ? occ_tile_decompress(ls.keep) : occ_tile_step(gsrc, opt, ls.keep),
                                     static_lds, ls.max_segs * kSeg * 2);
    if (mode == kModeDecompress) {
        tile_kernel<kModeDecompress, kGradDense, kOptAdam, kExpandThreads><<<dim3((unsigned)ls.wgs), dim3(kExpandThreads), pad, s>>>(ls, inv_scale, k,
                                                                                                                          guard);
    } else if (opt == kOptAdam) {
        if (gsrc == kGradDense) SAMO_LAUNCH_TILE(kModeStep, kGradDense, kOptAdam);
        else if (gsrc == kGradC16) SAMO_LAUNCH_TILE(kModeStep, kGradC16, kOptAdam);
        else SAMO_LAUNCH_TILE(kModeStep, kGradC32, kOptAdam);
    } else {
        if (gsrc == kGradDense) SAMO_LAUNCH_TILE(kModeStep, kGradDense, kOptSgd);
        else if (gsrc == kGradC16) SAMO_LAUNCH_TILE(kModeStep, kGradC16, kOptSgd);
        else SAMO_LAUNCH_TILE(kModeStep, kGradC32, kOptSgd);
    }
    return hipGetLastError();
}

int single_layer_tile_segs(int64_t n, int64_t nnz, bool dense, bool dense_fp32)
{
    if (dense || n <= 0) return 1;
    const double per_seg = (double)kSegCost + (double)kNnzCost * (double)kSeg * ((double)nnz / (double)n);
    const int64_t cost = tile_cost_for(n, nnz, dense_fp32);
    const int segs = (int)((double)cost / per_seg + 0.5);
    return segs < 1 ? 1 : (segs > tile_cost_segs(cost) ? tile_cost_segs(cost) : segs);
}

hipError_t launch_plan_write(const PlanBatch &batch, const PlanTables &t, hipStream_t s)
{
    plan_write_kernel<<<dim3(1), dim3(64), 0, s>>>(batch, t);
    return hipGetLastError();
}

hipError_t launch_plan_records(const PlanTables &t, int num_layers, int64_t ntiles, int64_t nchunks, int64_t tile_cost,
                               hipStream_t s)
{
    if (ntiles > 0)
        build_tile_recs_kernel<<<dim3((unsigned)ceil_div(ntiles, kThreads)), dim3(kThreads), 0, s>>>(
            t.layers, t.tile_start, num_layers, ntiles, tile_cost, tile_cost_segs(tile_cost), t.tiles);
    if (nchunks > 0)
        build_chunk_recs_kernel<<<dim3((unsigned)ceil_div(nchunks, kThreads)), dim3(kThreads), 0, s>>>(
            t.chunk_start, num_layers, nchunks, t.chunks);
    return hipGetLastError();
}

static int occ_tile_step_fp32(float keep)
{
    // a tile carries twice the dense bytes of the fp16 path: half the workgroups (measured at 90 %:
    // 6.1 TB/s with 3 per CU, 5.6 with 2, 5.0 with 4; at 95 %, where a tile is larger still, 6.3 with 2
    // against 6.0 with 3)
    return knob(SAMO_KNOB_OCC_TILE_STEP32, keep < (float)kSparseKeep ? 2 : 3);
}

hipError_t launch_tile_fp32(const LaunchSet &ls, float factor, const OptK &k, const GuardK &guard, hipStream_t s)
{
    if (ls.wgs <= 0) return hipSuccess;
    if (ls.max_segs < 1 || ls.max_segs > kMaxTileSegs) return hipErrorInvalidValue;
    const int pad = tile_lds_request(occ_tile_step_fp32(ls.keep), 0, ls.max_segs * kSeg * 4);
    tile_fp32_kernel<kTileThreads><<<dim3((unsigned)ls.wgs), dim3(kTileThreads), pad, s>>>(ls, factor, k, guard);
    return hipGetLastError();
}

hipError_t launch_gather(int out, int src, const LaunchSet &ls, float inv_scale, int accumulate,
                         StatPartial *partials, hipStream_t s)
{
    if (ls.wgs <= 0) return hipSuccess;
    if (partials && ls.layers && out == kOutNone && (src == kGradC16 || src == kGradC32)) {
        const int64_t per_xcd = ceil_div(ls.wgs, (int64_t)8);
        const dim3 run_grid((unsigned)(8 * ceil_div(per_xcd, (int64_t)kStatRun)));
        if (src == kGradC16) stats_compressed_kernel<kGradC16><<<run_grid, dim3(kFlatThreads), 0, s>>>(ls, inv_scale, partials);
        else stats_compressed_kernel<kGradC32><<<run_grid, dim3(kFlatThreads), 0, s>>>(ls, inv_scale, partials);
        return hipGetLastError();
    }
    const dim3 grid((unsigned)ls.wgs), block(kFlatThreads);
    const int pad = lds_pad_for(occ_flat_gather(out, src, ls.keep, partials != nullptr), 2 * kChunk * 4);   // static: the exchange areas
    if (out == kOutF32) gather_kernel<kOutF32><<<grid, block, pad, s>>>(ls, src, inv_scale, accumulate, partials);
    else if (out == kOutF16) gather_kernel<kOutF16><<<grid, block, pad, s>>>(ls, src, inv_scale, accumulate, partials);
    else gather_kernel<kOutNone><<<grid, block, pad, s>>>(ls, src, inv_scale, accumulate, partials);
    return hipGetLastError();
}

hipError_t launch_flat_step(int opt, const LaunchSet &ls, const OptK &k, const GuardK &guard, hipStream_t s)
{
    if (ls.wgs <= 0) return hipSuccess;
    const dim3 grid((unsigned)ls.wgs), block(kFlatThreads);
    const int g_flat_pad = lds_pad_for(occ_flat_step(), 0);
    if (opt == kOptAdam) flat_step_kernel<kOptAdam><<<grid, block, g_flat_pad, s>>>(ls, k, guard);
    else flat_step_kernel<kOptSgd><<<grid, block, g_flat_pad, s>>>(ls, k, guard);
    return hipGetLastError();
}

int64_t stats_workspace_partials(int64_t gather_wgs)
{
    return ceil_div(gather_wgs, 8) * 8 + kStatReduceGrid;
}

// Sums the partials a gather launch of `gather_wgs` workgroups left in `partials` (which must hold
// stats_workspace_partials(gather_wgs) entries) into *out: one level when there are few, else a
// first level of kStatReduceGrid workgroups that writes behind the partials.
hipError_t launch_stats_finalize(StatPartial *partials, int64_t gather_wgs, samo_grad_stats *out, hipStream_t s)
{
    const int64_t slots = ceil_div(gather_wgs, 8) * 8;
    if (slots <= 4 * kStatReduceGrid) {
        stats_finalize_kernel<<<dim3(1), dim3(kFinalizeThreads), 0, s>>>(partials, slots, (unsigned)gather_wgs, out);
    } else {
        const int64_t per = ceil_div(slots, (int64_t)kStatReduceGrid);
        const int64_t grid = ceil_div(slots, per);
        stats_reduce_kernel<<<dim3((unsigned)grid), dim3(kReduceThreads), 0, s>>>(partials, slots, (unsigned)gather_wgs,
                                                                                 per, partials + slots);
        stats_finalize_kernel<<<dim3(1), dim3(kFinalizeThreads), 0, s>>>(partials + slots, grid, 0u, out);
    }
    return hipGetLastError();
}

hipError_t launch_copy(void *dst, const void *src, int64_t bytes, hipStream_t s)
{
    const int64_t nvec = bytes / 16;
    const int64_t wgs = ceil_div(nvec, (int64_t)kThreads);
    if (wgs > 0)
        copy_kernel<<<dim3((unsigned)wgs), dim3(kThreads), 0, s>>>(reinterpret_cast<uint4 *>(dst),
                                                                  reinterpret_cast<const uint4 *>(src), nvec);
    return hipGetLastError();
}

}  // namespace samo
