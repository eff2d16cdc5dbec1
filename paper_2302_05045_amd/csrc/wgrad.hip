// Weight gradient of a fully connected layer written straight into the compressed gradient
// (Section III-C compresses each layer's dense fp16 gradient as soon as the backward pass has
// produced it; the paper's closing discussion of the compute overhead names fusing that
// compression into the backward kernels as the way to remove it).  dW = dY^T X is a dense
// contraction over the tokens: MFMA 32x32x16 fp16 with fp32 accumulation, operands staged through
// LDS; the epilogue rounds each accumulator once to fp16 — the value the dense gradient tensor
// would have held — and stores only the entries the layer's index keeps.  The dense gradient is
// never written to or read back from HBM.
#include <cstdlib>

#include "common.h"

namespace samo {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// Workgroup tile: 128 rows of dW (features of dY) by 256 columns (features of X) — wide along the
// direction in which the index runs, so that a row of the tile owns one contiguous run of idx —
// four waves as 2 x 2, each 64 x 128 = 2 x 4 MFMA blocks (128 accumulator registers per lane,
// two workgroups per compute unit).  32 tokens per stage, two stages in LDS.
constexpr int kWgOut = 128;
constexpr int kWgIn = 256;
constexpr int kWgTok = 32;
constexpr int kWgThreads = 256;
constexpr int kRowBytes = kWgTok * 2 + 8;                    // one feature's 32 tokens, padded: see stage_offset
constexpr int kStageBytes = (kWgIn + kWgOut) * kRowBytes;    // X rows, then dY rows
constexpr int kEpiRows = 64;                                 // rows of dW staged per epilogue pass
constexpr int kEpiPitch = kWgIn + 8;                         // halves; +8 spreads a column of 32 rows over the banks
constexpr int kOperandBytes = 2 * kStageBytes;
constexpr int kEpiBytes = kEpiRows * kEpiPitch * 2;
constexpr int kWgLdsBytes = kOperandBytes > kEpiBytes ? kOperandBytes : kEpiBytes;
static_assert(kWgLdsBytes + kWgOut * 2 * 4 <= 65536, "static LDS");
static_assert(kWgThreads == 256 && kWgIn == 256 && kWgOut == 128 && kWgTok == 32, "the thread-to-block maps below assume this shape");

// LDS image of a stage: row = feature (X: 0..255, dY: 256..383), 32 tokens = 64 bytes in a pitch
// of 72.  18 banks per row: a fragment read (32 lanes, 32 consecutive rows, 8 bytes each, twice)
// touches every bank once, and a store of 8 rows x 64 bytes whose rows are 8 (or 4) apart touches
// every bank twice — both the least possible.  Rows are 8-byte aligned only, so operands are
// read as pairs of 8-byte words.
__device__ __forceinline__ int stage_offset(int row, int chunk)
{
    return row * kRowBytes + (chunk << 4);
}

__device__ __forceinline__ half8 read_fragment(const unsigned char *p)
{
    const uint2 a = *reinterpret_cast<const uint2 *>(p);
    const uint2 b = *reinterpret_cast<const uint2 *>(p + 8);
    const uint4 q = make_uint4(a.x, a.y, b.x, b.y);
    return __builtin_bit_cast(half8, q);
}

struct WgradArgs {
    const _Float16 *dy;      // tokens x out
    const _Float16 *x;       // tokens x in
    int64_t tokens;
    int out, in;
    const int32_t *idx;
    const int32_t *seg_ptr;
    int64_t nnz;
    void *gc;                // fp32 or fp16, by the kernel's OUT
    float inv_scale;
    int accumulate;
    int tiles_in;
    int64_t tiles;
    int map;
};

template <int OUT>
__global__ void __launch_bounds__(kWgThreads, 2) wgrad_kernel(const WgradArgs A)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds[kWgLdsBytes];
    __shared__ int bounds[2 * kWgOut];

    // Workgroups are dealt round-robin to the 8 XCDs: give each XCD a contiguous run of tiles so
    // that the tiles sharing operand panels, and neighbouring runs of idx, meet in one L2.
    const int64_t per_xcd = (A.tiles + 7) / 8;
    const int64_t tile = A.map == 0 ? (int64_t)blockIdx.x : (int64_t)(blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (tile >= A.tiles) return;
    int row0, col0;
    if (A.map == 2) {                                        // out-tiles fastest
        const int tiles_out = (int)(A.tiles / A.tiles_in);
        row0 = (int)(tile % tiles_out) * kWgOut;
        col0 = (int)(tile / tiles_out) * kWgIn;
    } else {
        row0 = (int)(tile / A.tiles_in) * kWgOut;            // first row of dW (feature of dY)
        col0 = (int)(tile % A.tiles_in) * kWgIn;             // first column of dW (feature of X)
    }

    const int t = threadIdx.x;
    const int wave = t >> 6, lane = t & 63;
    const int kg = lane & 7;          // which 4 tokens of the stage this thread moves
    const int ml = lane >> 3;         // which feature block within the wave's share
    const int64_t n = (int64_t)A.out * A.in;

    // This thread's end of one row's run of idx (threads 0..127: start, 128..255: end), found by
    // bisection inside the segment seg_ptr names.  The probes ride along with the main loop, one
    // per stage, so that their latency costs nothing; what is left afterwards is finished there.
    int s_lo = 0, s_hi = 0, s_key = 0;
    {
        const int r = row0 + (t & (kWgOut - 1));
        if (r < A.out) {
            const int c = t < kWgOut ? col0 : (col0 + kWgIn < A.in ? col0 + kWgIn : A.in);
            const int64_t p = (int64_t)r * A.in + c;
            if (p >= n) s_lo = s_hi = (int)A.nnz;
            else if (!A.idx) s_lo = s_hi = (int)p;           // unpruned layer: position k is element k
            else {
                s_lo = A.seg_ptr[p / kSeg];
                s_hi = A.seg_ptr[p / kSeg + 1];
                s_key = (int)p;
            }
        }
    }

    // Global -> register -> LDS movers.  X: an 8-feature x 4-token block per thread (four 16-byte
    // loads), dY: a 4-feature x 4-token block (four 8-byte loads); both transposed in registers so
    // that LDS holds, per feature, tokens contiguously — what an MFMA operand lane needs.
    // Addresses are a uniform per-stage base plus a 32-bit offset per lane that never changes.
    // Features past the matrix are never gathered: their loads are only moved to a valid address.
    const int xf = col0 + (wave * 8 + ml) * 8;               // first X feature of the block
    const int yf = row0 + (wave * 8 + ml) * 4;               // first dY feature of the block
    uint32_t xoff[4], yoff[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        xoff[j] = ((uint32_t)(kg * 4 + j) * (uint32_t)A.in + (uint32_t)(xf < A.in ? xf : 0)) * 2u;
        yoff[j] = ((uint32_t)(kg * 4 + j) * (uint32_t)A.out + (uint32_t)(yf < A.out ? yf : 0)) * 2u;
    }
    const unsigned char *xbase = reinterpret_cast<const unsigned char *>(A.x);
    const unsigned char *ybase = reinterpret_cast<const unsigned char *>(A.dy);
    const int64_t xstage = (int64_t)kWgTok * A.in * 2, ystage = (int64_t)kWgTok * A.out * 2;   // bytes per stage
    struct Regs {
        uint4 x[4];
        uint2 y[4];
    };
    auto load_full_stage = [&](Regs &q, int64_t stage) {
        const unsigned char *xs = xbase + stage * xstage, *ys = ybase + stage * ystage;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            q.x[j] = *reinterpret_cast<const uint4 *>(xs + xoff[j]);
            q.y[j] = *reinterpret_cast<const uint2 *>(ys + yoff[j]);
        }
    };
    // The last stage when the token count is not a multiple of 32: rows past the end are read
    // from the last token and cleared, so that they add nothing.
    auto load_tail_stage = [&](Regs &q, int64_t stage) {
        const unsigned char *xs = xbase + stage * xstage, *ys = ybase + stage * ystage;
        const int rows = (int)(A.tokens - stage * kWgTok);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int row = kg * 4 + j;
            const uint32_t keep = row < rows ? 0xffffffffu : 0u;
            const uint32_t back = row < rows ? 0u : (uint32_t)(row - (rows - 1));
            const uint4 xv = *reinterpret_cast<const uint4 *>(xs + (xoff[j] - back * (uint32_t)A.in * 2u));
            const uint2 yv = *reinterpret_cast<const uint2 *>(ys + (yoff[j] - back * (uint32_t)A.out * 2u));
            q.x[j] = make_uint4(xv.x & keep, xv.y & keep, xv.z & keep, xv.w & keep);
            q.y[j] = make_uint2(yv.x & keep, yv.y & keep);
        }
    };
    const int64_t full_stages = A.tokens / kWgTok;
    const int64_t stages = (A.tokens + kWgTok - 1) / kWgTok;    // none: dW = 0
    auto load_stage = [&](Regs &q, int64_t stage) {
        if (stage < full_stages) load_full_stage(q, stage);
        else load_tail_stage(q, stage);
    };
    // Two fp16 lanes of two registers into one: the low halves, or the high halves.
    auto pack_lo = [](uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x05040100u); };
    auto pack_hi = [](uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); };
    auto store_stage = [&](const Regs &q, unsigned char *stage) {
        {
            const uint32_t d[4][4] = {{q.x[0].x, q.x[1].x, q.x[2].x, q.x[3].x}, {q.x[0].y, q.x[1].y, q.x[2].y, q.x[3].y},
                                      {q.x[0].z, q.x[1].z, q.x[2].z, q.x[3].z}, {q.x[0].w, q.x[1].w, q.x[2].w, q.x[3].w}};
            unsigned char *dst = stage + (wave * 8 + ml) * 8 * kRowBytes + kg * 8;
#pragma unroll
            for (int e = 0; e < 4; ++e) {                    // features 2e and 2e+1: tokens 0,1 | 2,3 of the block
                *reinterpret_cast<uint2 *>(dst + (2 * e) * kRowBytes) = make_uint2(pack_lo(d[e][0], d[e][1]), pack_lo(d[e][2], d[e][3]));
                *reinterpret_cast<uint2 *>(dst + (2 * e + 1) * kRowBytes) = make_uint2(pack_hi(d[e][0], d[e][1]), pack_hi(d[e][2], d[e][3]));
            }
        }
        {
            const uint32_t d[2][4] = {{q.y[0].x, q.y[1].x, q.y[2].x, q.y[3].x}, {q.y[0].y, q.y[1].y, q.y[2].y, q.y[3].y}};
            unsigned char *dst = stage + (kWgIn + (wave * 8 + ml) * 4) * kRowBytes + kg * 8;
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                *reinterpret_cast<uint2 *>(dst + (2 * e) * kRowBytes) = make_uint2(pack_lo(d[e][0], d[e][1]), pack_lo(d[e][2], d[e][3]));
                *reinterpret_cast<uint2 *>(dst + (2 * e + 1) * kRowBytes) = make_uint2(pack_hi(d[e][0], d[e][1]), pack_hi(d[e][2], d[e][3]));
            }
        }
    };

    // MFMA roles: the A operand (rows of a 32 x 32 block) takes X features, the B operand
    // (columns) takes dY features, so that a lane ends up with 4 consecutive columns of one row
    // of dW per accumulator quad.
    const int wo = wave & 1, wi = wave >> 1;
    const int l32 = lane & 31, khalf = lane >> 5;
    f32x16 acc[2][4];
#pragma unroll
    for (int bo = 0; bo < 2; ++bo)
#pragma unroll
        for (int bi = 0; bi < 4; ++bi)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[bo][bi][r] = 0.f;
    auto multiply_stage = [&](const unsigned char *cur) {
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            const int chunk = kk * 2 + khalf;
            half8 xa[4], yb[2];
#pragma unroll
            for (int bi = 0; bi < 4; ++bi) xa[bi] = read_fragment(cur + stage_offset(wi * 128 + bi * 32 + l32, chunk));
#pragma unroll
            for (int bo = 0; bo < 2; ++bo)
                yb[bo] = read_fragment(cur + stage_offset(kWgIn + wo * 64 + bo * 32 + l32, chunk));
#pragma unroll
            for (int bo = 0; bo < 2; ++bo)
#pragma unroll
                for (int bi = 0; bi < 4; ++bi)
                    acc[bo][bi] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa[bi], yb[bo], acc[bo][bi], 0, 0, 0);
        }
    };
    // One bisection probe: issued with a stage's loads, resolved after that stage's arithmetic.
    int s_mid = 0, s_val = 0;
    bool s_open = false;
    auto probe_issue = [&]() {
        s_open = s_lo < s_hi;
        s_mid = (s_lo + s_hi) >> 1;
        if (s_open) s_val = A.idx[s_mid];
    };
    auto probe_resolve = [&]() {
        if (s_open) {
            if (s_val < s_key) s_lo = s_mid + 1;
            else s_hi = s_mid;
        }
    };

    // Main loop: two LDS stages, the next stage's loads in flight during a stage's arithmetic, one
    // barrier per stage; written out for the two stages so that every LDS offset is a constant.
    unsigned char *const buf0 = lds, *const buf1 = lds + kStageBytes;
    Regs q;
    if (stages > 0) {
        load_stage(q, 0);
        store_stage(q, buf0);
    }
    __syncthreads();
    auto step = [&](const unsigned char *cur, unsigned char *nxt, int64_t next_stage) {
        const bool more = next_stage < stages;
        if (more) load_stage(q, next_stage);
        probe_issue();
        multiply_stage(cur);
        if (more) store_stage(q, nxt);
        probe_resolve();
        __syncthreads();
    };
    for (int64_t st = 0; st < stages; ++st) step((st & 1) ? buf1 : buf0, (st & 1) ? buf0 : buf1, st + 1);
    while (s_lo < s_hi) {
        probe_issue();
        probe_resolve();
    }

    // Epilogue, 64 rows of dW per pass (the two waves that own them write, everyone gathers):
    // accumulators -> fp16 image in LDS -> the kept entries of each row.  A half wave takes 8 rows
    // of a pass and fetches their index runs together before it touches the image.
    bounds[t] = s_lo;
    _Float16 *img = reinterpret_cast<_Float16 *>(lds);
    const int hw = t >> 5;
    constexpr int kRowsPerHalfWave = kEpiRows / 8;
#pragma unroll 1
    for (int pass = 0; pass < 2; ++pass) {
        if (wo == pass) {
#pragma unroll
            for (int bo = 0; bo < 2; ++bo)
#pragma unroll
                for (int bi = 0; bi < 4; ++bi)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        half4 h;
#pragma unroll
                        for (int e = 0; e < 4; ++e) h[e] = (_Float16)acc[bo][bi][q * 4 + e];   // round to nearest even
                        const int col = wi * 128 + bi * 32 + q * 8 + khalf * 4;
                        *reinterpret_cast<half4 *>(img + (bo * 32 + l32) * kEpiPitch + col) = h;
                    }
        }
        __syncthreads();
        int lo[kRowsPerHalfWave], hi[kRowsPerHalfWave], longest = 0;
#pragma unroll
        for (int it = 0; it < kRowsPerHalfWave; ++it) {
            const int trow = pass * kEpiRows + it * 8 + hw;
            lo[it] = bounds[trow];
            hi[it] = bounds[kWgOut + trow];
            longest = hi[it] - lo[it] > longest ? hi[it] - lo[it] : longest;
        }
        for (int off = l32; off - l32 < longest; off += 32) {
            int pos[kRowsPerHalfWave];
#pragma unroll
            for (int it = 0; it < kRowsPerHalfWave; ++it) {
                const int k = lo[it] + off;
                pos[it] = k < hi[it] ? (A.idx ? A.idx[k] : k) : -1;
            }
#pragma unroll
            for (int it = 0; it < kRowsPerHalfWave; ++it) {
                if (pos[it] < 0) continue;
                const int k = lo[it] + off;
                const int rl = it * 8 + hw;
                const int64_t base = (int64_t)(row0 + pass * kEpiRows + rl) * A.in + col0;
                const _Float16 v = img[rl * kEpiPitch + (int)(pos[it] - base)];
                if (OUT == kOutF32) {
                    reinterpret_cast<float *>(A.gc)[k] = (float)v * A.inv_scale;
                } else {
                    _Float16 *dst = reinterpret_cast<_Float16 *>(A.gc) + k;
                    *dst = A.accumulate ? (_Float16)(*dst + v) : v;
                }
            }
        }
        __syncthreads();
    }
}

}  // namespace

hipError_t launch_wgrad(int out_kind, const _Float16 *dy, const _Float16 *x, int64_t tokens, int64_t out, int64_t in,
                        const int32_t *idx, const int32_t *seg_ptr, int64_t nnz, void *gc, float inv_scale,
                        int accumulate, hipStream_t s)
{
    if (out <= 0 || in <= 0 || nnz <= 0) return hipSuccess;
    WgradArgs a;
    a.dy = dy; a.x = x; a.tokens = tokens; a.out = (int)out; a.in = (int)in;
    a.idx = idx; a.seg_ptr = seg_ptr; a.nnz = nnz; a.gc = gc; a.inv_scale = inv_scale; a.accumulate = accumulate;
    a.tiles_in = (int)ceil_div(in, kWgIn);
    a.tiles = ceil_div(out, kWgOut) * a.tiles_in;
    static const int map = getenv("SAMO_WGRAD_MAP") ? atoi(getenv("SAMO_WGRAD_MAP")) : 1;
    a.map = map;
    const unsigned grid = (unsigned)(ceil_div(a.tiles, 8) * 8);
    if (out_kind == kOutF32) wgrad_kernel<kOutF32><<<dim3(grid), dim3(kWgThreads), 0, s>>>(a);
    else wgrad_kernel<kOutF16><<<dim3(grid), dim3(kWgThreads), 0, s>>>(a);
    return hipGetLastError();
}

}  // namespace samo
