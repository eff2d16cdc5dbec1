// Weight gradient of a fully connected layer written straight into the compressed gradient
// (Section III-C compresses each layer's dense fp16 gradient as soon as the backward pass has
// produced it; Section VI-C, on the compute overhead of that compression, names fusing that
// compression into the backward kernels as the way to remove it).  dW = dY^T X is a dense
// contraction over the tokens: MFMA 32x32x16 fp16 with fp32 accumulation, operands staged through
// LDS; the epilogue rounds each accumulator once to fp16 — the value the dense gradient tensor
// would have held — and stores only the entries the layer's index keeps.  The dense gradient is
// never written to or read back from HBM.
#include <atomic>
#include <cstdlib>

#include "common.h"

namespace samo {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// Workgroup tile, large shape: 256 rows of dW (features of dY) by 256 columns (features of X), 8
// waves as 4 x 2, each 64 x 128 = 2 x 4 MFMA blocks (128 accumulator registers per lane, two waves
// per SIMD, one workgroup per CU).  32 tokens per stage, two stages in LDS, the loads of two
// further stages in flight in registers: per stage a thread moves one 8-feature x 4-token block
// (16 registers; the first half of the threads move X, the rest dY).  Small shape, for layers
// whose large tiles would leave compute units idle: 128 x 128 by 4 waves of 64 x 64, three
// workgroups per CU; it tops out at 0.6 of the large shape's rate (a third more LDS bytes per
// MFMA, twice the operand traffic) but is twice as fast on a 1024 x 4096 layer (64 large tiles).
// Measured on MI355X against the alternatives that were built and dropped: a 128 x 256 tile by 4
// waves, two workgroups per compute unit, with one stage of loads in flight (all its registers
// allow) reaches 0.6 of the large shape's rate at every layer size; the same 256 x 256 tile by 4
// waves of 128 x 128 (256 accumulators, one wave per SIMD, a third less LDS traffic) reaches 0.9
// — a lone wave per SIMD leaves its LDS stores, barrier and first fragment reads of every stage
// uncovered.
constexpr int kWgTok = 32;
constexpr int kRowBytes = kWgTok * 2 + 8;                    // one feature's 32 tokens, padded: see stage_offset
constexpr int kEpiRows = 128;                                // rows of dW staged per epilogue pass: two wave rows

// A tile shape: WO x WI waves, each BO x BI blocks of 32 x 32.  Every thread moves exactly one
// 8-feature block per stage and finds exactly one bound of the epilogue, so the tile's rows and
// columns together must equal the thread count.
template <int WO_, int WI_, int BO_, int BI_>
struct TileShape {
    static constexpr int WO = WO_, WI = WI_, BO = BO_, BI = BI_;
    static constexpr int kOut = WO * BO * 32;                // rows of dW per workgroup (features of dY)
    static constexpr int kIn = WI * BI * 32;                 // columns of dW per workgroup (features of X)
    static constexpr int kThreads = WO * WI * 64;
    static constexpr int kStageBytes = (kIn + kOut) * kRowBytes;     // X rows, then dY rows
    static constexpr int kLdsBytes = 2 * kStageBytes;
    static constexpr int kEpiPitch = kIn + 8;                // halves; +8 spreads a column of 32 rows over the banks
    static_assert(kIn + kOut == kThreads && 2 * kOut == kThreads, "one block to move and one bound to find per thread");
    static_assert(2 * BO * 32 == kEpiRows && WO % 2 == 0, "an epilogue pass is the rows of two wave rows");
    static_assert(kLdsBytes >= kEpiRows * kEpiPitch * 2, "the epilogue image reuses the operand stages");
    static_assert(kOut % 64 == 0 && kThreads % 32 == 0 && kEpiRows % (kThreads / 32) == 0, "epilogue row split");
};
using BigTile = TileShape<4, 2, 2, 4>;      // 256 x 256, 8 waves of 64 x 128: 128 accumulator registers, one workgroup per CU
using SmallTile = TileShape<2, 2, 2, 2>;    // 128 x 128, 4 waves of 64 x 64: layers whose 256 x 256 tiles would leave CUs idle
constexpr int64_t kSmallTileBelow = 65;     // 256 x 256 tiles of a layer below which the small shape is used (measured)

// LDS image of a stage: row = feature (X rows first, then dY rows), 32 tokens = 64 bytes in a pitch
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
};

struct Block8x4 {
    uint4 r[4];      // 4 tokens x 8 features
};

__device__ __forceinline__ uint32_t pack_lo16(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x05040100u); }
__device__ __forceinline__ uint32_t pack_hi16(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); }

// Writes the block as 8 feature rows of 4 tokens each.
__device__ __forceinline__ void store_block(const Block8x4 &q, unsigned char *dst)
{
    const uint32_t d[4][4] = {{q.r[0].x, q.r[1].x, q.r[2].x, q.r[3].x}, {q.r[0].y, q.r[1].y, q.r[2].y, q.r[3].y},
                              {q.r[0].z, q.r[1].z, q.r[2].z, q.r[3].z}, {q.r[0].w, q.r[1].w, q.r[2].w, q.r[3].w}};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        *reinterpret_cast<uint2 *>(dst + (2 * e) * kRowBytes) = make_uint2(pack_lo16(d[e][0], d[e][1]), pack_lo16(d[e][2], d[e][3]));
        *reinterpret_cast<uint2 *>(dst + (2 * e + 1) * kRowBytes) = make_uint2(pack_hi16(d[e][0], d[e][1]), pack_hi16(d[e][2], d[e][3]));
    }
}

template <int OUT, typename T>
__global__ void __launch_bounds__(T::kThreads, 2) wgrad_kernel(const WgradArgs A)
{
    constexpr int kWgOut = T::kOut, kWgIn = T::kIn, kStageBytes = T::kStageBytes, kEpiPitch = T::kEpiPitch;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    __shared__ int bounds[2 * kWgOut];

    // Workgroups are dealt round-robin to the 8 XCDs: give each XCD a contiguous run of tiles so
    // that the tiles sharing operand panels, and neighbouring runs of idx, meet in one L2.
    const int64_t per_xcd = (A.tiles + 7) / 8;
    const int64_t tile = (int64_t)(blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (tile >= A.tiles) return;
    // Within the run, tiles go down groups of 4 tile rows before they go across: the 32 tiles an
    // XCD works on at a time then share about 4 + 8 operand panels rather than 1 + 32.
    const int tiles_out = (int)(A.tiles / A.tiles_in);
    const int group = (int)(tile / (4 * A.tiles_in));
    const int in_group = (int)(tile - (int64_t)group * 4 * A.tiles_in);
    const int group_rows = tiles_out - group * 4 < 4 ? tiles_out - group * 4 : 4;
    const int row0 = (group * 4 + in_group % group_rows) * kWgOut;   // first row of dW (feature of dY)
    const int col0 = (in_group / group_rows) * kWgIn;                // first column of dW (feature of X)

    const int t = threadIdx.x;
    const int wave = t >> 6, lane = t & 63;
    const int kg = lane & 7;          // which 4 tokens of the stage this thread moves
    const int64_t n = (int64_t)A.out * A.in;

    // A row of the tile owns one contiguous run of idx.  This thread finds one end of one row's
    // run (the first half of the threads: the start, the rest: the end) by bisection inside the segment that
    // seg_ptr names; the probes ride along with the main loop.
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

    // Mover role of this thread: one 8-feature x 4-token block of X (the first waves) or of dY (the
    // rest) per stage: four 16-byte loads, transposed in registers so that LDS holds, per feature,
    // tokens contiguously — what an MFMA operand lane needs.  Addresses are a uniform per-stage
    // base plus a 32-bit offset per lane that never changes.  Features past the matrix are never
    // gathered: their loads are only moved to a valid address.
    const bool moves_dy = t >= kWgIn;                                      // uniform within a wave
    const int blk = (moves_dy ? t - kWgIn : t) >> 3;                       // which 8 features of its operand's tile
    const int features = moves_dy ? A.out : A.in;
    const int f = (moves_dy ? row0 : col0) + blk * 8;
    const unsigned char *src = reinterpret_cast<const unsigned char *>(moves_dy ? A.dy : A.x);
    const int64_t stage_bytes = (int64_t)kWgTok * features * 2;
    uint32_t off[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) off[j] = ((uint32_t)(kg * 4 + j) * (uint32_t)features + (uint32_t)(f < features ? f : 0)) * 2u;
    const int lds_dst = ((moves_dy ? kWgIn : 0) + blk * 8) * kRowBytes + kg * 8;
    auto load_full = [&](Block8x4 &q, int64_t stage) {
        const unsigned char *sp = src + stage * stage_bytes;
#pragma unroll
        for (int j = 0; j < 4; ++j) q.r[j] = *reinterpret_cast<const uint4 *>(sp + off[j]);
    };
    // The last stage when the token count is not a multiple of 32: rows past the end are read
    // from the last token and cleared, so that they add nothing.
    auto load_tail = [&](Block8x4 &q, int64_t stage) {
        const unsigned char *sp = src + stage * stage_bytes;
        const int rows = (int)(A.tokens - stage * kWgTok);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int row = kg * 4 + j;
            const uint32_t keep = row < rows ? 0xffffffffu : 0u;
            const uint32_t back = row < rows ? 0u : (uint32_t)(row - (rows - 1));
            const uint4 v = *reinterpret_cast<const uint4 *>(sp + (off[j] - back * (uint32_t)features * 2u));
            q.r[j] = make_uint4(v.x & keep, v.y & keep, v.z & keep, v.w & keep);
        }
    };

    // MFMA roles: the A operand (rows of a 32 x 32 block) takes X features, the B operand
    // (columns) takes dY features, so that a lane ends up with 4 consecutive columns of one row
    // of dW per accumulator quad.  Both operands give a lane the same 8 tokens (lanes 0-31 the
    // first 8 of a group of 16, lanes 32-63 the rest), which is all the contraction needs.
    constexpr int BO = T::BO, BI = T::BI;
    const int wo = wave % T::WO, wi = wave / T::WO;
    const int l32 = lane & 31, khalf = lane >> 5;
    f32x16 acc[BO][BI];
#pragma unroll
    for (int bo = 0; bo < BO; ++bo)
#pragma unroll
        for (int bi = 0; bi < BI; ++bi)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[bo][bi][r] = 0.f;
    auto multiply_stage = [&](const unsigned char *cur) {
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            const int chunk = kk * 2 + khalf;
            half8 xa[BI], yb[BO];
#pragma unroll
            for (int bi = 0; bi < BI; ++bi) xa[bi] = read_fragment(cur + stage_offset((wi * BI + bi) * 32 + l32, chunk));
#pragma unroll
            for (int bo = 0; bo < BO; ++bo)
                yb[bo] = read_fragment(cur + stage_offset(kWgIn + (wo * BO + bo) * 32 + l32, chunk));
#pragma unroll
            for (int bo = 0; bo < BO; ++bo)
#pragma unroll
                for (int bi = 0; bi < BI; ++bi)
                    acc[bo][bi] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa[bi], yb[bo], acc[bo][bi], 0, 0, 0);
        }
    };

    // One bisection probe per pair of stages: issued right behind the loads of the pair's first
    // stage, used after the second stage has waited for those same loads — it never makes a
    // stage wait for loads younger than the ones it needs anyway.
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

    // Main loop over the full stages, written out for the two LDS stages and the two register
    // sets: while stage s is multiplied out of LDS, stage s+1 sits in (or is on its way to) one
    // register set and stage s+2 is being requested into the other.  Inside the loop every load
    // is unconditional, so that the wait before a store to LDS can leave exactly the younger
    // stage's loads outstanding; the last two or three stages run after it.
    unsigned char *const buf0 = lds, *const buf1 = lds + kStageBytes;
    const int64_t full = A.tokens / kWgTok;
    Block8x4 qa, qb;
    if (full >= 2) {
        load_full(qa, 0);
        load_full(qb, 1);
        store_block(qa, buf0 + lds_dst);
        __syncthreads();
        int64_t st = 0;
        for (; st + 3 < full; st += 2) {
            load_full(qa, st + 2);
            probe_issue();
            __builtin_amdgcn_sched_barrier(0);           // requests first, then the arithmetic that hides them
            multiply_stage(buf0);
            store_block(qb, buf1 + lds_dst);
            __syncthreads();
            load_full(qb, st + 3);
            __builtin_amdgcn_sched_barrier(0);
            multiply_stage(buf1);
            store_block(qa, buf0 + lds_dst);
            __builtin_amdgcn_sched_barrier(0);           // keep the probe's use behind the wait above
            probe_resolve();
            __syncthreads();
        }
        // stage st is in buf0, stage st+1 in qb; a third one remains when the count is odd
        const bool third = st + 2 < full;
        if (third) load_full(qa, st + 2);
        multiply_stage(buf0);
        store_block(qb, buf1 + lds_dst);
        __syncthreads();
        multiply_stage(buf1);
        if (third) store_block(qa, buf0 + lds_dst);
        __syncthreads();
        if (third) {
            multiply_stage(buf0);
            __syncthreads();
        }
    } else if (full == 1) {
        load_full(qa, 0);
        store_block(qa, buf0 + lds_dst);
        __syncthreads();
        multiply_stage(buf0);
        __syncthreads();
    }
    if (A.tokens > full * kWgTok) {                      // the partial last stage, on its own
        load_tail(qa, full);
        store_block(qa, buf0 + lds_dst);
        __syncthreads();
        multiply_stage(buf0);
        __syncthreads();
    }
    while (s_lo < s_hi) {                                // what the main loop left of the bisection
        const int mid = (s_lo + s_hi) >> 1;
        if (A.idx[mid] < s_key) s_lo = mid + 1;
        else s_hi = mid;
    }

    // Epilogue, 128 rows of dW per pass (the waves that own them write, everyone gathers):
    // accumulators -> fp16 image in LDS -> the kept entries of each row.  A half wave takes its
    // share of the rows of a pass and fetches their index runs together before it touches the image.
    bounds[t] = s_lo;
    _Float16 *img = reinterpret_cast<_Float16 *>(lds);
    const int hw = t >> 5;
    constexpr int kHalfWaves = T::kThreads / 32;
    constexpr int kRowsPerHalfWave = kEpiRows / kHalfWaves;
#pragma unroll 1
    for (int pass = 0; pass < T::WO / 2; ++pass) {
        if ((wo >> 1) == pass) {
#pragma unroll
            for (int bo = 0; bo < BO; ++bo)
#pragma unroll
                for (int bi = 0; bi < BI; ++bi)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        half4 h;
#pragma unroll
                        for (int e = 0; e < 4; ++e) h[e] = (_Float16)acc[bo][bi][q * 4 + e];   // round to nearest even
                        const int col = (wi * BI + bi) * 32 + q * 8 + khalf * 4;
                        *reinterpret_cast<half4 *>(img + ((wo & 1) * 64 + bo * 32 + l32) * kEpiPitch + col) = h;
                    }
        }
        __syncthreads();
        int lo[kRowsPerHalfWave], hi[kRowsPerHalfWave], longest = 0;
#pragma unroll
        for (int it = 0; it < kRowsPerHalfWave; ++it) {
            const int trow = pass * kEpiRows + it * kHalfWaves + hw;
            lo[it] = bounds[trow];
            hi[it] = bounds[kWgOut + trow];
            longest = hi[it] - lo[it] > longest ? hi[it] - lo[it] : longest;
        }
        for (int off_k = l32; off_k - l32 < longest; off_k += 32) {
            int pos[kRowsPerHalfWave];
#pragma unroll
            for (int it = 0; it < kRowsPerHalfWave; ++it) {
                const int k = lo[it] + off_k;
                pos[it] = k < hi[it] ? (A.idx ? A.idx[k] : k) : -1;
            }
#pragma unroll
            for (int it = 0; it < kRowsPerHalfWave; ++it) {
                if (pos[it] < 0) continue;
                const int k = lo[it] + off_k;
                const int rl = it * kHalfWaves + hw;
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


// ---------------------------------------------------------------------------------------------
// The kernel for layers of 65 tiles and more: the operands go global -> LDS without passing
// registers (global_load_lds_dwordx4: each lane names 16 bytes of global memory, the wave's
// 1 KiB lands contiguously in LDS at a base held in M0), in the layout they have in memory — per
// token, 256 features of X then 256 of dY — and the MFMA operands are formed by the transposing
// LDS read ds_read_b64_tr_b16: within each group of 16 lanes, lanes 4r .. 4r+3 name the 16
// features of token r (r = 0..3), and lane i receives feature i of those four tokens.  No
// transposes on the vector ALU and no registers for bytes in flight: three whole stages are on
// their way while a fourth is multiplied, by 8 waves of 64 x 128 (128 accumulators each, two
// waves per SIMD, so that one wave's LDS reads and barrier waits sit under the other's MFMAs).
// The compiler cannot know which LDS reads alias a copy in flight and would wait for all of
// them before every read, so the copies are issued from inline assembly and this kernel counts
// its outstanding copies itself: every stage issues exactly 4 per wave.
// Measured against the register-staged kernel above at 256 x 256 (FC1 of the 2.7B model, 2048
// tokens): 0.144 against 0.168 ms; with 4 waves of 128 x 128 and one wave per SIMD the same
// copies gave 0.167 ms.
#define LDS_AS __attribute__((address_space(3)))
typedef short short4v __attribute__((ext_vector_type(4)));
constexpr int kDmaRowBytes = 1024 + 64;                 // one token: 256 X features, 256 dY features, pad
constexpr int kDmaStageBytes = kWgTok * kDmaRowBytes;   // 34816
constexpr int kDmaStages = 4;
constexpr int kDmaLdsBytes = kDmaStages * kDmaStageBytes;
constexpr int kDmaThreads = 512;
constexpr int kDmaEpiPitch = 256 + 8;

__device__ __attribute__((aligned(16))) const unsigned char wgrad_zero_row[16] = {0};

__device__ __forceinline__ void dma16(const void *g, unsigned lds_byte_addr)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_byte_addr) : "memory");
}

// 8 tokens of one feature for an MFMA lane: two transposing reads of 4 tokens each.
__device__ __forceinline__ half8 read_tr_fragment(const unsigned char *p)
{
    const short4v a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS short4v *)(LDS_AS unsigned char *)p);
    const short4v b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS short4v *)(LDS_AS unsigned char *)(p + 4 * kDmaRowBytes));
    typedef short short8v __attribute__((ext_vector_type(8)));
    const short8v q = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
    return __builtin_bit_cast(half8, q);
}

template <int OUT>
__global__ void __launch_bounds__(kDmaThreads, 2) wgrad_dma_kernel(const WgradArgs A)
{
    constexpr int kWgOut = 256, kWgIn = 256;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    __shared__ int bounds[2 * kWgOut];

    const int64_t per_xcd = (A.tiles + 7) / 8;
    const int64_t tile = (int64_t)(blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (tile >= A.tiles) return;
    const int tiles_out = (int)(A.tiles / A.tiles_in);
    const int group = (int)(tile / (4 * A.tiles_in));
    const int in_group = (int)(tile - (int64_t)group * 4 * A.tiles_in);
    const int group_rows = tiles_out - group * 4 < 4 ? tiles_out - group * 4 : 4;
    const int row0 = (group * 4 + in_group % group_rows) * kWgOut;
    const int col0 = (in_group / group_rows) * kWgIn;

    const int t = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6), lane = t & 63;
    const int64_t n = (int64_t)A.out * A.in;

    // Thread t < 256 looks for the first kept position of tile row t, thread 256 + t for the first
    // one past the row's end inside the tile.
    int s_lo = 0, s_hi = 0, s_key = 0;
    {
        const int r = row0 + (t & (kWgOut - 1));
        if (r < A.out) {
            const int c = t < kWgOut ? col0 : (col0 + kWgIn < A.in ? col0 + kWgIn : A.in);
            const int64_t p = (int64_t)r * A.in + c;
            if (p >= n) s_lo = s_hi = (int)A.nnz;
            else if (!A.idx) s_lo = s_hi = (int)p;
            else {
                s_lo = A.seg_ptr[p / kSeg];
                s_hi = A.seg_ptr[p / kSeg + 1];
                s_key = (int)p;
            }
        }
    }

    // DMA role of a lane: lanes 0-31 fetch 8 features of X each, lanes 32-63 8 features of dY; one
    // instruction of a wave moves one token's row of the stage.  Wave w owns rows 4w .. 4w+3.  Rows
    // past the last token are copied from 16 bytes of zeros, so that every stage is 4 copies per
    // wave and the wait counts below hold for the partial last stage too.
    const bool is_y = lane >= 32;
    const int features = is_y ? A.out : A.in;
    const int f = (is_y ? row0 : col0) + (lane & 31) * 8;
    const int64_t row_bytes = (int64_t)features * 2;
    const unsigned char *gbase = reinterpret_cast<const unsigned char *>(is_y ? A.dy : A.x) + (int64_t)(f < features ? f : 0) * 2;
    const unsigned lds_base = (unsigned)(size_t)(LDS_AS unsigned char *)lds;
    const int64_t stages = (A.tokens + kWgTok - 1) / kWgTok;
    auto issue_stage = [&](int64_t s) {
        const unsigned dst = lds_base + (unsigned)(s % kDmaStages) * kDmaStageBytes + (unsigned)(wave * 4) * kDmaRowBytes;
        const int64_t token = s * kWgTok + wave * 4;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            dma16(token + i < A.tokens ? gbase + (token + i) * row_bytes : wgrad_zero_row, dst + i * kDmaRowBytes);
    };

    const int wo = wave & 3, wi = wave >> 2;
    const int l32 = lane & 31;
    f32x16 acc[2][4];
#pragma unroll
    for (int bo = 0; bo < 2; ++bo)
#pragma unroll
        for (int bi = 0; bi < 4; ++bi)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[bo][bi][r] = 0.f;
    // lane address of a transposing read inside a stage: group of 16 lanes g, lane j of the group
    // reads token 8*(g>>1) + (j>>2), features 16*(g&1) + 4*(j&3) .. +3 of a 32-feature block
    const int g16 = lane >> 4, j16 = lane & 15;
    const int tr_off = (8 * (g16 >> 1) + (j16 >> 2)) * kDmaRowBytes + (16 * (g16 & 1) + 4 * (j16 & 3)) * 2;
    const int x_off = tr_off + (wi * 128) * 2, y_off = tr_off + 512 + (wo * 64) * 2;
    auto multiply_stage = [&](const unsigned char *cur) {
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            half8 xa[4], yb[2];
#pragma unroll
            for (int bi = 0; bi < 4; ++bi) xa[bi] = read_tr_fragment(cur + x_off + kk * 16 * kDmaRowBytes + bi * 64);
#pragma unroll
            for (int bo = 0; bo < 2; ++bo) yb[bo] = read_tr_fragment(cur + y_off + kk * 16 * kDmaRowBytes + bo * 64);
#pragma unroll
            for (int bo = 0; bo < 2; ++bo)
#pragma unroll
                for (int bi = 0; bi < 4; ++bi)
                    acc[bo][bi] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa[bi], yb[bo], acc[bo][bi], 0, 0, 0);
        }
    };

    // Three stages requested ahead, one barrier per stage.  At the top of stage s the copies of
    // stages s+1 and s+2 may still be outstanding (8 per wave), those of stage s may not.
    for (int64_t s = 0; s < 3 && s < stages; ++s) issue_stage(s);
    // The bounds are searched while those first stages are on their way.  First a guess by
    // interpolation inside the segment (kept elements spread evenly over it would put the bound
    // at lo + (hi - lo) * offset / 1024) and a look at the 8 entries around it — on masks without
    // structure that settles it in one round trip; then plain bisection of whatever is left.
    if (s_lo < s_hi) {
        const int guess = s_lo + (int)(((int64_t)(s_hi - s_lo) * (s_key & (kSeg - 1))) >> 10);
        int w0 = guess - 4 > s_lo ? guess - 4 : s_lo;
        if (w0 + 8 > s_hi) w0 = s_hi - 8 > s_lo ? s_hi - 8 : s_lo;
        const int wn = s_hi - w0 < 8 ? s_hi - w0 : 8;
        int v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = A.idx[w0 + (i < wn ? i : wn - 1)];
        int below = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) below += (i < wn && v[i] < s_key) ? 1 : 0;
        if (below == 0) s_hi = w0;                          // the bound is at or before the window
        else if (below == wn) s_lo = w0 + wn;                // at or after its end
        else s_lo = s_hi = w0 + below;                    // inside
    }
    while (s_lo < s_hi) {
        const int mid = (s_lo + s_hi) >> 1;
        if (A.idx[mid] < s_key) s_lo = mid + 1;
        else s_hi = mid;
    }
    bounds[t] = s_lo;
    for (int64_t s = 0; s < stages; ++s) {
        const int64_t younger = stages - 1 - s < 2 ? stages - 1 - s : 2;
        if (younger == 2) asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)" ::: "memory");
        else if (younger == 1) asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (s + 3 < stages) issue_stage(s + 3);
        multiply_stage(lds + (s % kDmaStages) * kDmaStageBytes);
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __syncthreads();

    _Float16 *img = reinterpret_cast<_Float16 *>(lds);
    const int hw = t >> 5, khalf = lane >> 5;
    constexpr int kPassRows = 128;
    constexpr int kRowsPerHalfWave = kPassRows / 16;
#pragma unroll 1
    for (int pass = 0; pass < 2; ++pass) {
        if ((wo >> 1) == pass) {
#pragma unroll
            for (int bo = 0; bo < 2; ++bo)
#pragma unroll
                for (int bi = 0; bi < 4; ++bi)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        half4 h;
#pragma unroll
                        for (int e = 0; e < 4; ++e) h[e] = (_Float16)acc[bo][bi][q * 4 + e];
                        const int col = wi * 128 + bi * 32 + q * 8 + khalf * 4;
                        *reinterpret_cast<half4 *>(img + ((wo & 1) * 64 + bo * 32 + l32) * kDmaEpiPitch + col) = h;
                    }
        }
        __syncthreads();
        int lo[kRowsPerHalfWave], hi[kRowsPerHalfWave], longest = 0;
#pragma unroll
        for (int it = 0; it < kRowsPerHalfWave; ++it) {
            const int trow = pass * kPassRows + it * 16 + hw;
            lo[it] = bounds[trow];
            hi[it] = bounds[kWgOut + trow];
            longest = hi[it] - lo[it] > longest ? hi[it] - lo[it] : longest;
        }
        for (int off_k = l32; off_k - l32 < longest; off_k += 32) {
            int pos[kRowsPerHalfWave];
#pragma unroll
            for (int it = 0; it < kRowsPerHalfWave; ++it) {
                const int k = lo[it] + off_k;
                pos[it] = k < hi[it] ? (A.idx ? A.idx[k] : k) : -1;
            }
#pragma unroll
            for (int it = 0; it < kRowsPerHalfWave; ++it) {
                if (pos[it] < 0) continue;
                const int k = lo[it] + off_k;
                const int rl = it * 16 + hw;
                const int64_t base = (int64_t)(row0 + pass * kPassRows + rl) * A.in + col0;
                const _Float16 v = img[rl * kDmaEpiPitch + (int)(pos[it] - base)];
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

template <typename T>
hipError_t launch_shape(int out_kind, WgradArgs a, int64_t out, int64_t in, hipStream_t s)
{
    // The LDS size above 64 KiB is a per-device attribute of the kernel: set once per device.
    static std::atomic<uint64_t> configured{0};
    int device = 0;
    if (hipError_t e = hipGetDevice(&device)) return e;
    const uint64_t bit = 1ull << (device & 63);
    if (!(configured.load(std::memory_order_acquire) & bit)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&wgrad_kernel<kOutF32, T>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, T::kLdsBytes);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(&wgrad_kernel<kOutF16, T>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, T::kLdsBytes);
        if (e != hipSuccess) return e;
        configured.fetch_or(bit, std::memory_order_release);
    }
    a.tiles_in = (int)ceil_div(in, T::kIn);
    a.tiles = ceil_div(out, T::kOut) * a.tiles_in;
    const unsigned grid = (unsigned)(ceil_div(a.tiles, 8) * 8);   // whole rounds of the 8 XCDs; the surplus exits at once
    if (out_kind == kOutF32) wgrad_kernel<kOutF32, T><<<dim3(grid), dim3(T::kThreads), T::kLdsBytes, s>>>(a);
    else wgrad_kernel<kOutF16, T><<<dim3(grid), dim3(T::kThreads), T::kLdsBytes, s>>>(a);
    return hipGetLastError();
}

hipError_t launch_dma(int out_kind, WgradArgs a, int64_t out, int64_t in, hipStream_t s)
{
    constexpr int kBytes = kDmaLdsBytes;
    static std::atomic<uint64_t> configured{0};
    int device = 0;
    if (hipError_t e = hipGetDevice(&device)) return e;
    const uint64_t bit = 1ull << (device & 63);
    if (!(configured.load(std::memory_order_acquire) & bit)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&wgrad_dma_kernel<kOutF32>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kBytes);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(&wgrad_dma_kernel<kOutF16>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kBytes);
        if (e != hipSuccess) return e;
        configured.fetch_or(bit, std::memory_order_release);
    }
    a.tiles_in = (int)ceil_div(in, 256);
    a.tiles = ceil_div(out, 256) * a.tiles_in;
    const unsigned grid = (unsigned)(ceil_div(a.tiles, 8) * 8);
    if (out_kind == kOutF32) wgrad_dma_kernel<kOutF32><<<dim3(grid), dim3(kDmaThreads), kBytes, s>>>(a);
    else wgrad_dma_kernel<kOutF16><<<dim3(grid), dim3(kDmaThreads), kBytes, s>>>(a);
    return hipGetLastError();
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
    a.tiles_in = 0; a.tiles = 0;
    const int64_t big_tiles = ceil_div(out, BigTile::kOut) * ceil_div(in, BigTile::kIn);
    const char *forced = getenv("SAMO_WGRAD_TILE");           // tuning and test aid, read per call: 128, 256 or 512 (= 256, copies straight to LDS)
    const int force = forced ? atoi(forced) : 0;
    const bool small = force == 128 || (force != 256 && force != 512 && big_tiles < kSmallTileBelow);
    if (small) return launch_shape<SmallTile>(out_kind, a, out, in, s);
    if (force == 256) return launch_shape<BigTile>(out_kind, a, out, in, s);
    return launch_dma(out_kind, a, out, in, s);
}

}  // namespace samo
