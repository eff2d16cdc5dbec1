// Expansion, gradient compression, compressed Adam and the fused optimizer phase
// (Section III-C of the paper) as HBM-streaming kernels for gfx950.
//
// Dense side (fp16 w and g, N elements): a workgroup owns one aligned tile of
// kTile elements.  The new fp16 weights of the tile are assembled in LDS — zero
// filled, then the kept values dropped in at their tile-relative positions — and
// leave as whole 16-byte vectors, so HBM never sees a partial-line write and the
// explicit zeros of the pruned positions cost no extra pass.
// Compressed side (idx, p, m, v, gc; nnz elements): the tile's slice is
// [seg_ptr[first segment], seg_ptr[last segment + 1]); consecutive lanes take
// consecutive compressed elements, so every access is a contiguous run.
// Gradients are read at the kept positions only; with ascending indices the
// lanes of a wave fall into a handful of neighbouring cache lines.
//
// There is no matrix contraction anywhere on this path: it is bound by HBM
// bandwidth, and each byte is touched once.
#include "common.h"

namespace samo {
namespace {

__device__ __forceinline__ float half_bits_to_float(uint16_t h)
{
    return (float)__builtin_bit_cast(_Float16, h);          // exact, subnormals honoured
}

// fp32 -> fp16, round to nearest even.  The empty asm makes x opaque, so the conversion always
// starts from the fp32 value that is also stored as the master parameter; without it the compiler
// folds the last fma of the Adam update and this conversion into one v_fma_mixlo_f16, which rounds
// the exact fma result once to fp16 and so differs from fp16(fp32(p)) on double-rounding cases.
__device__ __forceinline__ uint16_t float_to_half_bits(float x)
{
    asm("" : "+v"(x));
    return __builtin_bit_cast(uint16_t, (_Float16)x);
}

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void store16(void *dst, const uint4 &v)
{
#if SAMO_NT & 1
    __builtin_nontemporal_store((u32x4){v.x, v.y, v.z, v.w}, reinterpret_cast<u32x4 *>(dst));
#else
    *reinterpret_cast<uint4 *>(dst) = v;
#endif
}

__device__ __forceinline__ void store_f32(float *dst, float v)
{
#if SAMO_NT & 2
    __builtin_nontemporal_store(v, dst);
#else
    *dst = v;
#endif
}

typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void store_f4(float *dst, const float4 &v)
{
#if SAMO_NT & 8
    __builtin_nontemporal_store((f32x4){v.x, v.y, v.z, v.w}, reinterpret_cast<f32x4 *>(dst));
#else
    *reinterpret_cast<float4 *>(dst) = v;
#endif
}

template <typename T>
__device__ __forceinline__ T load_stream(const T *src)
{
#if SAMO_NT & 4
    return __builtin_nontemporal_load(src);
#else
    return *src;
#endif
}

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

// ------------------------------------------------------------------ tile kernels
enum { kModeDecompress = 0, kModeFused = 1 };

// Dense (unpruned) layer: identity index, plain elementwise pass over the tile.
template <int MODE>
__device__ __forceinline__ void dense_tile(const samo_layer &L, int64_t base, int len, float inv_scale,
                                           const AdamK &k)
{
    const int tid = threadIdx.x;
    float *__restrict__ P = L.p + base;
    uint16_t *__restrict__ W = L.w + base;
    const int nvec = len / 8;
    for (int o = tid; o < nvec; o += kTileThreads) {
        float4 p0 = reinterpret_cast<const float4 *>(P)[2 * o];
        float4 p1 = reinterpret_cast<const float4 *>(P)[2 * o + 1];
        float pv[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
        if (MODE == kModeFused) {
            float *__restrict__ M = L.m + base;
            float *__restrict__ V = L.v + base;
            const uint4 gq = reinterpret_cast<const uint4 *>(L.g + base)[o];
            const uint32_t gw[4] = {gq.x, gq.y, gq.z, gq.w};
            float4 m0 = reinterpret_cast<const float4 *>(M)[2 * o];
            float4 m1 = reinterpret_cast<const float4 *>(M)[2 * o + 1];
            float4 v0 = reinterpret_cast<const float4 *>(V)[2 * o];
            float4 v1 = reinterpret_cast<const float4 *>(V)[2 * o + 1];
            float mv[8] = {m0.x, m0.y, m0.z, m0.w, m1.x, m1.y, m1.z, m1.w};
            float vv[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint16_t gb = (uint16_t)(gw[e >> 1] >> (16 * (e & 1)));
                adam_update(pv[e], mv[e], vv[e], half_bits_to_float(gb) * inv_scale, k);
            }
            reinterpret_cast<float4 *>(P)[2 * o] = make_float4(pv[0], pv[1], pv[2], pv[3]);
            reinterpret_cast<float4 *>(P)[2 * o + 1] = make_float4(pv[4], pv[5], pv[6], pv[7]);
            reinterpret_cast<float4 *>(M)[2 * o] = make_float4(mv[0], mv[1], mv[2], mv[3]);
            reinterpret_cast<float4 *>(M)[2 * o + 1] = make_float4(mv[4], mv[5], mv[6], mv[7]);
            reinterpret_cast<float4 *>(V)[2 * o] = make_float4(vv[0], vv[1], vv[2], vv[3]);
            reinterpret_cast<float4 *>(V)[2 * o + 1] = make_float4(vv[4], vv[5], vv[6], vv[7]);
        }
        uint32_t hw[4];
#pragma unroll
        for (int q = 0; q < 4; ++q)
            hw[q] = (uint32_t)float_to_half_bits(pv[2 * q]) | ((uint32_t)float_to_half_bits(pv[2 * q + 1]) << 16);
        reinterpret_cast<uint4 *>(W)[o] = make_uint4(hw[0], hw[1], hw[2], hw[3]);
    }
    for (int e = nvec * 8 + tid; e < len; e += kTileThreads) {      // ragged end of the layer
        float pe = P[e];
        if (MODE == kModeFused) {
            float me = L.m[base + e], ve = L.v[base + e];
            adam_update(pe, me, ve, half_bits_to_float(L.g[base + e]) * inv_scale, k);
            P[e] = pe;
            L.m[base + e] = me;
            L.v[base + e] = ve;
        }
        W[e] = float_to_half_bits(pe);
    }
}

template <int MODE>
__device__ __forceinline__ void sparse_tile(const samo_layer &L, int tile, int64_t base, int len, float inv_scale,
                                            const AdamK &k, uint16_t *lds_w, uint16_t *lds_g)
{
    const int tid = threadIdx.x;
    uint4 *l4 = reinterpret_cast<uint4 *>(lds_w);
#if SAMO_GLDS
    if (MODE == kModeFused) {                 // stage the tile's dense gradient through LDS, fully coalesced
        constexpr int NV = kTile / 8 / kTileThreads;
        uint4 gq[NV];
        const uint4 *gsrc = reinterpret_cast<const uint4 *>(L.g + base);
        const int nvec_g = (len + 7) / 8;     // a 16-byte aligned buffer always holds whole vectors? no: guard below
#pragma unroll
        for (int q = 0; q < NV; ++q) {
            const int o = tid + q * kTileThreads;
            gq[q] = make_uint4(0u, 0u, 0u, 0u);
            if (o * 8 + 8 <= len) gq[q] = gsrc[o];
            else if (o < nvec_g) {
                uint16_t tmp[8] = {0, 0, 0, 0, 0, 0, 0, 0};
                for (int e = 0; e < 8; ++e) if (o * 8 + e < len) tmp[e] = L.g[base + o * 8 + e];
                gq[q] = make_uint4(tmp[0] | (tmp[1] << 16), tmp[2] | (tmp[3] << 16), tmp[4] | (tmp[5] << 16),
                                   tmp[6] | (tmp[7] << 16));
            }
        }
#pragma unroll
        for (int q = 0; q < NV; ++q) reinterpret_cast<uint4 *>(lds_g)[tid + q * kTileThreads] = gq[q];
    }
#endif
#pragma unroll
    for (int o = tid; o < kTile / 8; o += kTileThreads) l4[o] = make_uint4(0u, 0u, 0u, 0u);

    const int64_t nseg = (L.n + kSeg - 1) / kSeg;
    const int64_t s0 = (int64_t)tile * kSegsPerTile;
    const int64_t s1 = (s0 + kSegsPerTile < nseg) ? s0 + kSegsPerTile : nseg;
    const int c0 = L.seg_ptr[s0];
    const int c1 = L.seg_ptr[s1];
    __syncthreads();

    // the tile's slice of the compressed arrays; at most kTile elements, so slice-relative
    // offsets fit an int even when c0 is close to 2^31
    const int cnt = c1 - c0;
    const int32_t *__restrict__ IDX = L.idx + c0;
    float *__restrict__ P = L.p + c0;
    float *__restrict__ M = L.m + c0;
    float *__restrict__ V = L.v + c0;
    const uint16_t *__restrict__ G = L.g;
    const int ibase = (int)base;             // a layer's flat size fits int32

    constexpr int U = SAMO_U;
    for (int r0 = tid; r0 < cnt; r0 += U * kTileThreads) {
        int j[U];
        float pp[U], mm[U], vv[U];
        uint16_t gb[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int r = r0 + u * kTileThreads;
            j[u] = ibase; pp[u] = 0.f; mm[u] = 0.f; vv[u] = 0.f; gb[u] = 0;
            if (r < cnt) {
                j[u] = load_stream(IDX + r);
                pp[u] = load_stream(P + r);
                if (MODE == kModeFused) { mm[u] = load_stream(M + r); vv[u] = load_stream(V + r); }
            }
        }
        if (MODE == kModeFused) {
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (r0 + u * kTileThreads < cnt) gb[u] = SAMO_GLDS ? lds_g[j[u] - ibase] : G[j[u]];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int r = r0 + u * kTileThreads;
            if (r < cnt) {
                if (MODE == kModeFused) {
                    adam_update(pp[u], mm[u], vv[u], half_bits_to_float(gb[u]) * inv_scale, k);
                    store_f32(P + r, pp[u]);
                    store_f32(M + r, mm[u]);
                    store_f32(V + r, vv[u]);
                }
                lds_w[j[u] - ibase] = float_to_half_bits(pp[u]);
            }
        }
    }
    __syncthreads();

    uint16_t *__restrict__ W = L.w + base;
    const int nvec = len / 8;
    for (int o = tid; o < nvec; o += kTileThreads) store16(reinterpret_cast<uint4 *>(W) + o, l4[o]);
    for (int e = nvec * 8 + tid; e < len; e += kTileThreads) W[e] = lds_w[e];
}

template <int MODE, bool BATCHED>
__global__ void __launch_bounds__(kTileThreads)
tile_kernel(const samo_layer one, const samo_layer *__restrict__ layers, const WgRec *__restrict__ recs,
            float inv_scale, const AdamK k)
{
    __shared__ __attribute__((aligned(16))) uint16_t lds_w[kTile];
#if SAMO_GLDS
    __shared__ __attribute__((aligned(16))) uint16_t lds_g_buf[MODE == kModeFused ? kTile : 8];
    uint16_t *lds_g = lds_g_buf;
#else
    uint16_t *lds_g = nullptr;
#endif
    samo_layer L;
    int tile;
    if (BATCHED) {
        const WgRec r = recs[blockIdx.x];
        L = layers[r.layer];
        tile = r.local;
    } else {
        L = one;
        tile = blockIdx.x;
    }
    const int64_t base = (int64_t)tile * kTile;
    const int64_t rest = L.n - base;
    const int len = rest < kTile ? (int)rest : kTile;
    if (L.seg_ptr == nullptr)                 // dense (unpruned) layer
        dense_tile<MODE>(L, base, len, inv_scale, k);
    else
        sparse_tile<MODE>(L, tile, base, len, inv_scale, k, lds_w, lds_g);
}

// ------------------------------------------------------------------ flat kernels over the compressed arrays
template <bool BATCHED>
__global__ void __launch_bounds__(kFlatThreads)
gather_kernel(const samo_layer one, const samo_layer *__restrict__ layers, const WgRec *__restrict__ recs,
              float inv_scale)
{
    samo_layer L;
    int64_t chunk;
    if (BATCHED) {
        const WgRec r = recs[blockIdx.x];
        L = layers[r.layer];
        chunk = r.local;
    } else {
        L = one;
        chunk = blockIdx.x;
    }
    const int64_t nnz = L.nnz;
    const uint16_t *__restrict__ G = L.g;
    float *__restrict__ GC = L.gc;
#pragma unroll
    for (int it = 0; it < kChunk / (4 * kFlatThreads); ++it) {
        const int64_t i = chunk * kChunk + ((int64_t)it * kFlatThreads + threadIdx.x) * 4;
        if (L.idx == nullptr) {                                   // dense layer: identity index
            if (i + 4 <= nnz) {
                const uint2 q = *reinterpret_cast<const uint2 *>(G + i);
                float4 o;
                o.x = half_bits_to_float((uint16_t)q.x) * inv_scale;
                o.y = half_bits_to_float((uint16_t)(q.x >> 16)) * inv_scale;
                o.z = half_bits_to_float((uint16_t)q.y) * inv_scale;
                o.w = half_bits_to_float((uint16_t)(q.y >> 16)) * inv_scale;
                *reinterpret_cast<float4 *>(GC + i) = o;
            } else {
                for (int64_t e = i; e < nnz; ++e) GC[e] = half_bits_to_float(G[e]) * inv_scale;
            }
        } else if (i + 4 <= nnz) {
            const int4 j = *reinterpret_cast<const int4 *>(L.idx + i);
            const uint16_t a = G[j.x], b = G[j.y], c = G[j.z], d = G[j.w];
            float4 o;
            o.x = half_bits_to_float(a) * inv_scale;
            o.y = half_bits_to_float(b) * inv_scale;
            o.z = half_bits_to_float(c) * inv_scale;
            o.w = half_bits_to_float(d) * inv_scale;
            store_f4(GC + i, o);
        } else {
            for (int64_t e = i; e < nnz; ++e) GC[e] = half_bits_to_float(G[L.idx[e]]) * inv_scale;
        }
    }
}

template <bool BATCHED>
__global__ void __launch_bounds__(kFlatThreads)
adam_kernel(const samo_layer one, const samo_layer *__restrict__ layers, const WgRec *__restrict__ recs,
            const AdamK k)
{
    samo_layer L;
    int64_t chunk;
    if (BATCHED) {
        const WgRec r = recs[blockIdx.x];
        L = layers[r.layer];
        chunk = r.local;
    } else {
        L = one;
        chunk = blockIdx.x;
    }
    const int64_t nnz = L.nnz;
    float *__restrict__ P = L.p;
    float *__restrict__ M = L.m;
    float *__restrict__ V = L.v;
    const float *__restrict__ GC = L.gc;
#if SAMO_ADAM_DWORD
    {
        constexpr int U = kChunk / kFlatThreads;
        float pp[U], mm[U], vv[U], gg[U];
        const int64_t i0 = chunk * kChunk + threadIdx.x;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = i0 + u * kFlatThreads;
            if (i < nnz) { pp[u] = P[i]; mm[u] = M[i]; vv[u] = V[i]; gg[u] = GC[i]; }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = i0 + u * kFlatThreads;
            if (i < nnz) {
                adam_update(pp[u], mm[u], vv[u], gg[u], k);
                P[i] = pp[u]; M[i] = mm[u]; V[i] = vv[u];
            }
        }
    }
#else
#pragma unroll
    for (int it = 0; it < kChunk / (4 * kFlatThreads); ++it) {
        const int64_t i = chunk * kChunk + ((int64_t)it * kFlatThreads + threadIdx.x) * 4;
        if (i + 4 <= nnz) {
            float4 p = *reinterpret_cast<const float4 *>(P + i);
            float4 m = *reinterpret_cast<const float4 *>(M + i);
            float4 v = *reinterpret_cast<const float4 *>(V + i);
            const float4 g = *reinterpret_cast<const float4 *>(GC + i);
            adam_update(p.x, m.x, v.x, g.x, k);
            adam_update(p.y, m.y, v.y, g.y, k);
            adam_update(p.z, m.z, v.z, g.z, k);
            adam_update(p.w, m.w, v.w, g.w, k);
            store_f4(P + i, p);
            store_f4(M + i, m);
            store_f4(V + i, v);
        } else {
            for (int64_t e = i; e < nnz; ++e) {
                float p = P[e], m = M[e], v = V[e];
                adam_update(p, m, v, GC[e], k);
                P[e] = p; M[e] = m; V[e] = v;
            }
        }
    }
#endif
}

// ------------------------------------------------------------------ diagnostic copy
constexpr int kCopyVecPerThread = 1;                              // 16 bytes per thread, 4 KiB per workgroup: the fastest shape measured

__global__ void __launch_bounds__(kThreads)
copy_kernel(uint4 *__restrict__ dst, const uint4 *__restrict__ src, int64_t nvec)
{
    const int64_t first = (int64_t)blockIdx.x * (kThreads * kCopyVecPerThread) + threadIdx.x;
    uint4 r[kCopyVecPerThread];
#pragma unroll
    for (int u = 0; u < kCopyVecPerThread; ++u) {
        const int64_t o = first + (int64_t)u * kThreads;
        r[u] = (o < nvec) ? src[o] : make_uint4(0u, 0u, 0u, 0u);
    }
#pragma unroll
    for (int u = 0; u < kCopyVecPerThread; ++u) {
        const int64_t o = first + (int64_t)u * kThreads;
        if (o < nvec) dst[o] = r[u];
    }
}

const AdamK kNoAdam = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0, 0};
const samo_layer kNoLayer = {0, 0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};

}  // namespace

hipError_t launch_decompress(const samo_layer &layer, hipStream_t s)
{
    const int64_t tiles = ceil_div(layer.n, kTile);
    if (tiles > 0)
        tile_kernel<kModeDecompress, false><<<dim3((unsigned)tiles), dim3(kTileThreads), 0, s>>>(layer, nullptr, nullptr,
                                                                                            1.f, kNoAdam);
    return hipGetLastError();
}

hipError_t launch_fused(const samo_layer &layer, float inv_scale, const AdamK &k, hipStream_t s)
{
    const int64_t tiles = ceil_div(layer.n, kTile);
    if (tiles > 0)
        tile_kernel<kModeFused, false><<<dim3((unsigned)tiles), dim3(kTileThreads), 0, s>>>(layer, nullptr, nullptr,
                                                                                       inv_scale, k);
    return hipGetLastError();
}

hipError_t launch_gather(const samo_layer &layer, float inv_scale, hipStream_t s)
{
    const int64_t chunks = ceil_div(layer.nnz, kChunk);
    if (chunks > 0)
        gather_kernel<false><<<dim3((unsigned)chunks), dim3(kFlatThreads), 0, s>>>(layer, nullptr, nullptr, inv_scale);
    return hipGetLastError();
}

hipError_t launch_adam(const samo_layer &layer, const AdamK &k, hipStream_t s)
{
    const int64_t chunks = ceil_div(layer.nnz, kChunk);
    if (chunks > 0)
        adam_kernel<false><<<dim3((unsigned)chunks), dim3(kFlatThreads), 0, s>>>(layer, nullptr, nullptr, k);
    return hipGetLastError();
}

hipError_t launch_decompress_batched(const samo_layer *d_layers, const WgRec *d_tiles, int64_t ntiles, hipStream_t s)
{
    if (ntiles > 0)
        tile_kernel<kModeDecompress, true><<<dim3((unsigned)ntiles), dim3(kTileThreads), 0, s>>>(kNoLayer, d_layers,
                                                                                            d_tiles, 1.f, kNoAdam);
    return hipGetLastError();
}

hipError_t launch_fused_batched(const samo_layer *d_layers, const WgRec *d_tiles, int64_t ntiles, float inv_scale,
                                const AdamK &k, hipStream_t s)
{
    if (ntiles > 0)
        tile_kernel<kModeFused, true><<<dim3((unsigned)ntiles), dim3(kTileThreads), 0, s>>>(kNoLayer, d_layers, d_tiles,
                                                                                       inv_scale, k);
    return hipGetLastError();
}

hipError_t launch_gather_batched(const samo_layer *d_layers, const WgRec *d_chunks, int64_t nchunks, float inv_scale,
                                 hipStream_t s)
{
    if (nchunks > 0)
        gather_kernel<true><<<dim3((unsigned)nchunks), dim3(kFlatThreads), 0, s>>>(kNoLayer, d_layers, d_chunks,
                                                                              inv_scale);
    return hipGetLastError();
}

hipError_t launch_adam_batched(const samo_layer *d_layers, const WgRec *d_chunks, int64_t nchunks, const AdamK &k,
                               hipStream_t s)
{
    if (nchunks > 0)
        adam_kernel<true><<<dim3((unsigned)nchunks), dim3(kFlatThreads), 0, s>>>(kNoLayer, d_layers, d_chunks, k);
    return hipGetLastError();
}

hipError_t launch_copy(void *dst, const void *src, int64_t bytes, hipStream_t s)
{
    const int64_t nvec = bytes / 16;
    const int64_t wgs = ceil_div(nvec, (int64_t)kThreads * kCopyVecPerThread);
    if (wgs > 0)
        copy_kernel<<<dim3((unsigned)wgs), dim3(kThreads), 0, s>>>(reinterpret_cast<uint4 *>(dst),
                                                                  reinterpret_cast<const uint4 *>(src), nvec);
    return hipGetLastError();
}

}  // namespace samo
