// Weight gradient of a fully connected layer written straight into the compressed gradient
// (Section III-C compresses each layer's dense fp16 gradient as soon as the backward pass has
// produced it; Section VI-C, on the compute overhead of that compression, names fusing that
// compression into the backward kernels as the way to remove it).  dW = dY^T X is a dense
// contraction over the tokens: MFMA 32x32x16 fp16 with fp32 accumulation, operands staged through
// LDS; the epilogue rounds each accumulator once to fp16 — the value the dense gradient tensor
// would have held — and stores only the entries the layer's index keeps.  The dense gradient is
// never written to or read back from HBM.
//
// How the operands travel.  They arrive tokens-outer (dY is tokens x out, X is tokens x in) and go
// global -> LDS without passing registers (global_load_lds_dwordx4: each lane names 16 bytes of
// global memory, the wave's 1 KiB lands contiguously in LDS at a base held in M0), in the layout
// they have in memory — per token, a run of X features then a run of dY features.  An MFMA lane
// wants 8 tokens of one feature; the transposing LDS read ds_read_b64_tr_b16 forms that: within
// each group of 16 lanes, lanes 4r .. 4r+3 name the 16 features of token r (r = 0..3), and lane i
// receives feature i of those four tokens.  No transposes on the vector ALU and no registers for
// bytes in flight: a ring of four stages, three on their way while the fourth is multiplied.
// The compiler cannot know which LDS reads alias a copy in flight and would wait for all of them
// before every read, so the copies are issued from inline assembly and the kernels count their
// outstanding copies themselves: every stage is exactly 4 copies per wave, the partial last stage
// included (rows past the last token are copied from a row of zeros).
//
// Two tile shapes, both 8 waves with two waves per SIMD — with one wave per SIMD nothing covers a
// wave's LDS reads and barrier waits, with two the other wave's MFMAs do (measured: 0.167 ms with
// 4 waves of 128 x 128, 0.144 ms with 8 waves of 64 x 128, FC1 of the GPT-3 2.7B shape at 2048
// tokens):
//   256 x 256, waves as 4 x 2 of 64 x 128 (128 accumulators), 32 tokens per stage;
//   128 x 128 for what is left of a layer after whole rounds of large tiles, where that is at
//   most half a round (so also for every layer of up to 128 large tiles): two
//   groups of four waves, each group covers the whole tile with 64 x 64 per wave (64 accumulators)
//   and multiplies half of the tokens of every 64-token stage; group 1 hands its sums to group 0
//   through LDS at the end.
#include <atomic>
#include <cstdlib>

#include "common.h"

namespace samo {
namespace {

#define LDS_AS __attribute__((address_space(3)))
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));

constexpr int kWgThreads = 512;
constexpr int kRowPitch = 1024 + 64;                 // an LDS row is one copy instruction's 1 KiB; the pad spreads rows over the banks
constexpr int kStageRows = 32;
constexpr int kStageBytes = kStageRows * kRowPitch;  // 34816
constexpr int kStages = 4;
constexpr int kLdsBytes = kStages * kStageBytes;     // 139264: one workgroup per CU
constexpr int kBigTile = 256, kBigTokens = 32;       // tokens per stage: one per LDS row
constexpr int kSmallTile = 128, kSmallTokens = 64;   // two per LDS row

// What a workgroup knows of the layer its tile belongs to.
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
};

// A launch: the 256 x 256 tiles of up to kWgradMaxJobs layers in one list, layer after layer
// (layer j owns tiles first_tile[j] .. first_tile[j+1] - 1, tiles_out[j] x tiles_in[j] of them);
// the launch's workgroups take tiles first .. first + tiles - 1 of that list, or, with quadrants
// set, four workgroups take the 128 x 128 quarters of each.
struct WgradBatch {
    WgradJob job[kWgradMaxJobs];
    int tiles_out[kWgradMaxJobs], tiles_in[kWgradMaxJobs];
    int64_t first_tile[kWgradMaxJobs + 1];
    int jobs;
    float inv_scale;
    int accumulate;
    int quadrants;
    int64_t first, tiles;
};

__device__ __attribute__((aligned(16))) const unsigned char wgrad_zero_row[16] = {0};

// One copy instruction: the wave's 64 x 16 bytes from the lanes' global addresses to LDS at
// lds_byte_addr + 16 * lane.  It writes M0, a register the compiler reserves and does not let an
// asm statement declare as clobbered; nothing else in these kernels makes the compiler use M0 (no
// register arrays indexed at run time, no other LDS-direct or GWS operation).
__device__ __forceinline__ void dma16(const void *g, unsigned lds_byte_addr)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_byte_addr) : "memory");
}

// 8 tokens of one feature for an MFMA lane: two transposing reads of 4 tokens (LDS rows) each.
__device__ __forceinline__ half8 read_tr_fragment(const unsigned char *p)
{
    const short4v a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS short4v *)(LDS_AS unsigned char *)p);
    const short4v b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS short4v *)(LDS_AS unsigned char *)(p + 4 * kRowPitch));
    const short8v q = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
    return __builtin_bit_cast(half8, q);
}

// Byte offset, inside a stage, of a lane's first transposing read for a 32-feature block that
// starts at byte 0 of the rows: group of 16 lanes g, lane j of the group reads LDS row
// 8*(g>>1) + (j>>2), features 16*(g&1) + 4*(j&3) .. +3.
__device__ __forceinline__ int tr_lane_offset(int lane)
{
    const int g = lane >> 4, j = lane & 15;
    return (8 * (g >> 1) + (j >> 2)) * kRowPitch + (16 * (g & 1) + 4 * (j & 3)) * 2;
}

// Workgroups are dealt round-robin to the 8 XCDs: each XCD gets a contiguous run of tiles so
// that the tiles sharing operand panels, and neighbouring runs of idx, meet in one L2.  Within
// the run, tiles go down groups of 4 tile rows before they go across: the 32 tiles an XCD works on
// at a time then share about 4 + 8 operand panels rather than 1 + 32.
// Returns false for a workgroup with nothing to do: the surplus of the last round, or a quarter
// that lies outside the matrix.
__device__ __forceinline__ bool tile_origin(const WgradBatch &B, WgradArgs &A, int &row0, int &col0)
{
    const int64_t blocks = B.quadrants ? B.tiles * 4 : B.tiles;
    const int64_t per_xcd = (blocks + 7) / 8;
    const int64_t local = (int64_t)(blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (local >= blocks) return false;
    const int64_t listed = B.first + (B.quadrants ? local >> 2 : local);
    int j = 0;
    while (j + 1 < B.jobs && listed >= B.first_tile[j + 1]) ++j;
    const WgradJob &J = B.job[j];
    A.dy = J.dy; A.x = J.x; A.tokens = J.tokens; A.out = J.out; A.in = J.in;
    A.idx = J.idx; A.seg_ptr = J.seg_ptr; A.nnz = J.nnz; A.gc = J.gc;
    A.inv_scale = B.inv_scale; A.accumulate = B.accumulate;
    const int64_t tile = listed - B.first_tile[j];
    const int tiles_out = B.tiles_out[j], tiles_in = B.tiles_in[j];
    const int group = (int)(tile / (4 * tiles_in));
    const int in_group = (int)(tile - (int64_t)group * 4 * tiles_in);
    const int group_rows = tiles_out - group * 4 < 4 ? tiles_out - group * 4 : 4;
    row0 = (group * 4 + in_group % group_rows) * kBigTile;   // first row of dW (feature of dY)
    col0 = (in_group / group_rows) * kBigTile;               // first column of dW (feature of X)
    if (B.quadrants) {
        row0 += (int)(local & 1) * kSmallTile;
        col0 += (int)((local >> 1) & 1) * kSmallTile;
    }
    return row0 < A.out && col0 < A.in;
}

// The kept entries of a tile row are a run of idx between two bounds: the first kept position at
// or after the row's first column in the tile, and the first one at or after the column where the
// tile ends.  A bound is searched in three steps with the tile's other work between them:
// bound_open reads the segment's range from seg_ptr, bound_window requests a few entries of idx
// where the bound should be, bound_settle decides.
struct Bound {
    int lo, hi, key;
};

__device__ __forceinline__ Bound bound_open(const WgradArgs &A, int row, int col)
{
    Bound b = {0, 0, 0};
    if (row >= A.out) return b;                                   // no such row: an empty run
    const int64_t p = (int64_t)row * A.in + (col < A.in ? col : A.in);
    if (p >= (int64_t)A.out * A.in) b.lo = b.hi = (int)A.nnz;
    else if (!A.idx) b.lo = b.hi = (int)p;                        // nothing pruned: position = entry
    else {
        b.lo = A.seg_ptr[p / kSeg];
        b.hi = A.seg_ptr[p / kSeg + 1];
        b.key = (int)p;
    }
    return b;
}

// First a guess by interpolation inside the segment (kept elements spread evenly over it would
// put the bound at lo + (hi - lo) * offset / 1024) and a look at the 8 entries around it — on
// masks without structure that settles it in one round trip; then bisection of what is left.
// The look is requested by bound_window and used by bound_settle, which a kernel calls after its
// main loop: the entries travel while the tile is multiplied.
struct Window {
    int w0, wn;
    int v[8];
};

__device__ __forceinline__ Window bound_window(const WgradArgs &A, const Bound &b)
{
    Window w;
    w.w0 = 0; w.wn = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) w.v[i] = 0;
    if (b.lo < b.hi) {
        const int guess = b.lo + (int)(((int64_t)(b.hi - b.lo) * (b.key & (kSeg - 1))) >> 10);
        w.w0 = guess - 4 > b.lo ? guess - 4 : b.lo;
        if (w.w0 + 8 > b.hi) w.w0 = b.hi - 8 > b.lo ? b.hi - 8 : b.lo;
        w.wn = b.hi - w.w0 < 8 ? b.hi - w.w0 : 8;
#pragma unroll
        for (int i = 0; i < 8; ++i) w.v[i] = A.idx[w.w0 + (i < w.wn ? i : w.wn - 1)];
    }
    return w;
}

__device__ __forceinline__ int bound_settle(const WgradArgs &A, Bound b, const Window &w)
{
    if (b.lo < b.hi) {
        int below = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) below += (i < w.wn && w.v[i] < b.key) ? 1 : 0;
        if (below == 0) b.hi = w.w0;                             // the bound is at or before the window
        else if (below == w.wn) b.lo = w.w0 + w.wn;              // at or after its end
        else b.lo = b.hi = w.w0 + below;                         // inside
    }
    while (b.lo < b.hi) {
        const int mid = (b.lo + b.hi) >> 1;
        if (A.idx[mid] < b.key) b.lo = mid + 1;
        else b.hi = mid;
    }
    return b.lo;
}

// The main loop both kernels share.  At the top of stage s the copies of stages s+1 and s+2 may
// still be outstanding (8 per wave), those of stage s may not; the barrier also tells every wave
// that the slot of stage s-1 has been read and may take stage s+3.  The 8 loads of bound_window
// sit between the copies of stages 2 and 3 in the same counter: they are older than every stage
// whose wait could mistake them for its own copies, so they can only make the waits of stages 0
// to 2 longer than needed, never shorter.
template <typename Issue, typename Multiply>
__device__ __forceinline__ void run_stages(int64_t stages, unsigned char *lds, Issue issue_stage, Multiply multiply_stage)
{
    for (int64_t s = 0; s < stages; ++s) {
        const int64_t younger = stages - 1 - s < 2 ? stages - 1 - s : 2;
        if (younger == 2) asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)" ::: "memory");
        else if (younger == 1) asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (s + 3 < stages) issue_stage(s + 3);
        multiply_stage(lds + (s % kStages) * kStageBytes);
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __syncthreads();
}

// Epilogue over the ROWS rows of a tile held as an fp16 image in LDS: each of the 16 half-waves
// takes every 16th row, all of them at once; per row, idx between the row's two bounds is read
// coalesced, the values are picked from the image and the compressed gradient is written
// coalesced.
template <int OUT, int ROWS>
__device__ __forceinline__ void gather_pass(const WgradArgs &A, const _Float16 *img, int pitch, const int *first, const int *last,
                                            int first_row, int col0)
{
    constexpr int kRows = ROWS / (kWgThreads / 32);
    const int hw = threadIdx.x >> 5, l32 = threadIdx.x & 31;
    int lo[kRows], hi[kRows], longest = 0;
#pragma unroll
    for (int it = 0; it < kRows; ++it) {
        lo[it] = first[it * 16 + hw];
        hi[it] = last[it * 16 + hw];
        longest = hi[it] - lo[it] > longest ? hi[it] - lo[it] : longest;
    }
    for (int off_k = l32; off_k - l32 < longest; off_k += 32) {
        int pos[kRows];
#pragma unroll
        for (int it = 0; it < kRows; ++it) {
            const int k = lo[it] + off_k;
            pos[it] = k < hi[it] ? (A.idx ? A.idx[k] : k) : -1;
        }
#pragma unroll
        for (int it = 0; it < kRows; ++it) {
            if (pos[it] < 0) continue;
            const int k = lo[it] + off_k;
            const int rl = it * 16 + hw;
            const int64_t base = (int64_t)(first_row + rl) * A.in + col0;
            const _Float16 v = img[rl * pitch + (int)(pos[it] - base)];
            if (OUT == kOutF32) {
                reinterpret_cast<float *>(A.gc)[k] = (float)v * A.inv_scale;
            } else {
                _Float16 *dst = reinterpret_cast<_Float16 *>(A.gc) + k;
                *dst = A.accumulate ? (_Float16)(*dst + v) : v;
            }
        }
    }
}

// 256 x 256 tile.  LDS row j of a stage: token j as 256 X features then 256 dY features.
template <int OUT>
__global__ void __launch_bounds__(kWgThreads, 2) wgrad_big_kernel(const WgradBatch B)
{
    constexpr int kTile = kBigTile, kEpiPitch = kTile + 8;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    __shared__ int bounds[2 * kTile];
    WgradArgs A;
    int row0, col0;
    if (!tile_origin(B, A, row0, col0)) return;

    const int t = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6), lane = t & 63;
    // thread t < 256: the first bound of tile row t; thread 256 + t: its second
    const Bound open = bound_open(A, row0 + (t & (kTile - 1)), t < kTile ? col0 : col0 + kTile);

    // Copy role of a lane: lanes 0-31 bring 8 features of X each, lanes 32-63 8 features of dY; one
    // instruction of a wave moves one token.  Wave w owns rows 4w .. 4w+3 of every stage.
    const bool is_y = lane >= 32;
    const int features = is_y ? A.out : A.in;
    const int f = (is_y ? row0 : col0) + (lane & 31) * 8;
    const int64_t row_bytes = (int64_t)features * 2;
    const unsigned char *gbase = reinterpret_cast<const unsigned char *>(is_y ? A.dy : A.x) + (int64_t)(f < features ? f : 0) * 2;
    const unsigned lds_base = (unsigned)(size_t)(LDS_AS unsigned char *)lds;
    const int64_t stages = (A.tokens + kBigTokens - 1) / kBigTokens;
    auto issue_stage = [&](int64_t s) {
        const unsigned dst = lds_base + (unsigned)(s % kStages) * kStageBytes + (unsigned)(wave * 4) * kRowPitch;
        const int64_t token = s * kBigTokens + wave * 4;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            dma16(token + i < A.tokens ? gbase + (token + i) * row_bytes : wgrad_zero_row, dst + i * kRowPitch);
    };

    const int wo = wave & 3, wi = wave >> 2;
    const int l32 = lane & 31, khalf = lane >> 5;
    f32x16 acc[2][4];
#pragma unroll
    for (int bo = 0; bo < 2; ++bo)
#pragma unroll
        for (int bi = 0; bi < 4; ++bi)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[bo][bi][r] = 0.f;
    const int x_off = tr_lane_offset(lane) + (wi * 128) * 2, y_off = tr_lane_offset(lane) + 512 + (wo * 64) * 2;
    auto multiply_stage = [&](const unsigned char *cur) {
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            half8 xa[4], yb[2];
#pragma unroll
            for (int bi = 0; bi < 4; ++bi) xa[bi] = read_tr_fragment(cur + x_off + kk * 16 * kRowPitch + bi * 64);
#pragma unroll
            for (int bo = 0; bo < 2; ++bo) yb[bo] = read_tr_fragment(cur + y_off + kk * 16 * kRowPitch + bo * 64);
#pragma unroll
            for (int bo = 0; bo < 2; ++bo)
#pragma unroll
                for (int bi = 0; bi < 4; ++bi)
                    acc[bo][bi] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa[bi], yb[bo], acc[bo][bi], 0, 0, 0);
        }
    };

    for (int64_t s = 0; s < 3 && s < stages; ++s) issue_stage(s);
    const Window window = bound_window(A, open);
    run_stages(stages, lds, issue_stage, multiply_stage);
    bounds[t] = bound_settle(A, open, window);

    _Float16 *img = reinterpret_cast<_Float16 *>(lds);
    static_assert(kTile * kEpiPitch * 2 <= kLdsBytes, "the whole tile's image fits in the stages");
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
                *reinterpret_cast<half4 *>(img + (wo * 64 + bo * 32 + l32) * kEpiPitch + col) = h;
            }
    __syncthreads();
    gather_pass<OUT, kTile>(A, img, kEpiPitch, bounds, bounds + kTile, row0, col0);
}

// 128 x 128 tile.  LDS row j of a stage: token j and token j + 32, each as 128 X features then
// 128 dY features; wave group g multiplies the tokens in slot g of the rows.
template <int OUT>
__global__ void __launch_bounds__(kWgThreads, 2) wgrad_small_kernel(const WgradBatch B)
{
    constexpr int kTile = kSmallTile, kEpiPitch = kTile + 8, kSumPitch = kTile + 4;
    static_assert(kTile * kSumPitch * 4 + kTile * kEpiPitch * 2 <= kLdsBytes, "group 1's sums and the image reuse the stages");
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    __shared__ int bounds[2 * kTile];
    WgradArgs A;
    int row0, col0;
    if (!tile_origin(B, A, row0, col0)) return;

    const int t = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6), lane = t & 63;
    // thread t < 128: the first bound of tile row t; thread 128 + t: its second; the rest: none
    const Bound open = t < 2 * kTile ? bound_open(A, row0 + (t & (kTile - 1)), t < kTile ? col0 : col0 + kTile) : Bound{0, 0, 0};

    // Copy role of a lane: token row + 32 * (lane >> 5); of its 32 lanes the first 16 bring 8
    // features of X each, the other 16 8 features of dY.  Wave w owns rows 4w .. 4w+3.
    const bool is_y = (lane & 16) != 0;
    const int features = is_y ? A.out : A.in;
    const int f = (is_y ? row0 : col0) + (lane & 15) * 8;
    const int64_t row_bytes = (int64_t)features * 2;
    const unsigned char *gbase = reinterpret_cast<const unsigned char *>(is_y ? A.dy : A.x) + (int64_t)(f < features ? f : 0) * 2;
    const int lane_token = wave * 4 + 32 * (lane >> 5);
    const unsigned lds_base = (unsigned)(size_t)(LDS_AS unsigned char *)lds;
    const int64_t stages = (A.tokens + kSmallTokens - 1) / kSmallTokens;
    auto issue_stage = [&](int64_t s) {
        const unsigned dst = lds_base + (unsigned)(s % kStages) * kStageBytes + (unsigned)(wave * 4) * kRowPitch;
        const int64_t token = s * kSmallTokens + lane_token;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            dma16(token + i < A.tokens ? gbase + (token + i) * row_bytes : wgrad_zero_row, dst + i * kRowPitch);
    };

    const int half = wave >> 2;                   // which 32 tokens of a stage
    const int wo = wave & 1, wi = (wave >> 1) & 1;
    const int l32 = lane & 31, khalf = lane >> 5;
    f32x16 acc[2][2];
#pragma unroll
    for (int bo = 0; bo < 2; ++bo)
#pragma unroll
        for (int bi = 0; bi < 2; ++bi)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[bo][bi][r] = 0.f;
    const int x_off = tr_lane_offset(lane) + half * 512 + (wi * 64) * 2, y_off = tr_lane_offset(lane) + half * 512 + 256 + (wo * 64) * 2;
    auto multiply_stage = [&](const unsigned char *cur) {
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            half8 xa[2], yb[2];
#pragma unroll
            for (int bi = 0; bi < 2; ++bi) xa[bi] = read_tr_fragment(cur + x_off + kk * 16 * kRowPitch + bi * 64);
#pragma unroll
            for (int bo = 0; bo < 2; ++bo) yb[bo] = read_tr_fragment(cur + y_off + kk * 16 * kRowPitch + bo * 64);
#pragma unroll
            for (int bo = 0; bo < 2; ++bo)
#pragma unroll
                for (int bi = 0; bi < 2; ++bi)
                    acc[bo][bi] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa[bi], yb[bo], acc[bo][bi], 0, 0, 0);
        }
    };

    for (int64_t s = 0; s < 3 && s < stages; ++s) issue_stage(s);
    const Window window = bound_window(A, open);
    run_stages(stages, lds, issue_stage, multiply_stage);
    const int closed = bound_settle(A, open, window);
    if (t < 2 * kTile) bounds[t] = closed;

    // group 1's sums -> LDS as fp32; group 0 adds them to its own, rounds once to fp16 and writes
    // the image behind them
    float *sums = reinterpret_cast<float *>(lds);
    _Float16 *img = reinterpret_cast<_Float16 *>(lds + kTile * kSumPitch * 4);
    if (half == 1) {
#pragma unroll
        for (int bo = 0; bo < 2; ++bo)
#pragma unroll
            for (int bi = 0; bi < 2; ++bi)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = wi * 64 + bi * 32 + q * 8 + khalf * 4;
                    *reinterpret_cast<float4 *>(sums + (wo * 64 + bo * 32 + l32) * kSumPitch + col) =
                        make_float4(acc[bo][bi][q * 4], acc[bo][bi][q * 4 + 1], acc[bo][bi][q * 4 + 2], acc[bo][bi][q * 4 + 3]);
                }
    }
    __syncthreads();
    if (half == 0) {
#pragma unroll
        for (int bo = 0; bo < 2; ++bo)
#pragma unroll
            for (int bi = 0; bi < 2; ++bi)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = wi * 64 + bi * 32 + q * 8 + khalf * 4;
                    const float4 o = *reinterpret_cast<const float4 *>(sums + (wo * 64 + bo * 32 + l32) * kSumPitch + col);
                    half4 h;                                                 // round to nearest even
                    h[0] = (_Float16)(acc[bo][bi][q * 4] + o.x);
                    h[1] = (_Float16)(acc[bo][bi][q * 4 + 1] + o.y);
                    h[2] = (_Float16)(acc[bo][bi][q * 4 + 2] + o.z);
                    h[3] = (_Float16)(acc[bo][bi][q * 4 + 3] + o.w);
                    *reinterpret_cast<half4 *>(img + (wo * 64 + bo * 32 + l32) * kEpiPitch + col) = h;
                }
    }
    __syncthreads();
    gather_pass<OUT, kTile>(A, img, kEpiPitch, bounds, bounds + kTile, row0, col0);
}

// What the matrix units sustain with nothing to fetch: every wave issues eight independent
// 32x32x16 fp16 MFMAs per iteration from registers (128 accumulators, the large tile's share), two
// waves to a SIMD as in the kernels above.  The operands are ordinary fp16 values (a few set
// mantissa and exponent bits, varying by lane), because the clock the chip holds under this load,
// and with it the rate, depends on how many bits toggle.  Each workgroup leaves one float.
__global__ void __launch_bounds__(kWgThreads, 2) mfma_rate_kernel(int64_t iters, float *__restrict__ sink)
{
    f32x16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    half8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (_Float16)(0.37f * (float)((int)(threadIdx.x % 7) + i) - 1.f);
        b[i] = (_Float16)(0.011f * (float)((int)(threadIdx.x % 5) + 2 * i) - 0.03f);
    }
    for (int64_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[i], 0, 0, 0);
    }
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) sum += acc[i][r];
    sum += __shfl_xor(sum, 32, 64);
    if (threadIdx.x == 0) sink[blockIdx.x] = sum;
}

// The LDS size above 64 KiB is a per-device attribute of a kernel: set once per device, where the
// device's number of compute units is read too.
hipError_t configure_once(int *cus)
{
    static std::atomic<uint64_t> configured{0};
    static int cus_of[64];
    int device = 0;
    if (hipError_t e = hipGetDevice(&device)) return e;
    const uint64_t bit = 1ull << (device & 63);
    if (!(configured.load(std::memory_order_acquire) & bit)) {
        const void *kernels[4] = {reinterpret_cast<const void *>(&wgrad_big_kernel<kOutF32>),
                                  reinterpret_cast<const void *>(&wgrad_big_kernel<kOutF16>),
                                  reinterpret_cast<const void *>(&wgrad_small_kernel<kOutF32>),
                                  reinterpret_cast<const void *>(&wgrad_small_kernel<kOutF16>)};
        for (const void *k : kernels)
            if (hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes)) return e;
        int n = 0;
        if (hipError_t e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, device)) return e;
        cus_of[device & 63] = n;
        configured.fetch_or(bit, std::memory_order_release);
    }
    *cus = cus_of[device & 63];
    return hipSuccess;
}

}  // namespace

hipError_t wgrad_configure(int *cus) { return configure_once(cus); }

hipError_t launch_mfma_rate(int64_t iters, float *sink, int workgroups, hipStream_t s)
{
    if (workgroups > 0) mfma_rate_kernel<<<dim3((unsigned)workgroups), dim3(kWgThreads), 0, s>>>(iters, sink);
    return hipGetLastError();
}

hipError_t launch_wgrad(int out_kind, const WgradJob *jobs, int count, float inv_scale, int accumulate, hipStream_t s)
{
    WgradBatch b;
    b.jobs = 0; b.inv_scale = inv_scale; b.accumulate = accumulate;
    b.first_tile[0] = 0;
    for (int j = 0; j < count && b.jobs < kWgradMaxJobs; ++j) {
        if (jobs[j].out <= 0 || jobs[j].in <= 0 || jobs[j].nnz <= 0) continue;     // nothing to write
        const int k = b.jobs++;
        b.job[k] = jobs[j];
        b.tiles_out[k] = (int)ceil_div(jobs[j].out, kBigTile);
        b.tiles_in[k] = (int)ceil_div(jobs[j].in, kBigTile);
        b.first_tile[k + 1] = b.first_tile[k] + (int64_t)b.tiles_out[k] * b.tiles_in[k];
    }
    if (b.jobs == 0) return hipSuccess;
    for (int k = b.jobs; k < kWgradMaxJobs; ++k) {
        b.job[k] = b.job[0]; b.tiles_out[k] = b.tiles_in[k] = 1; b.first_tile[k + 1] = b.first_tile[b.jobs];
    }
    int cus = 0;
    if (hipError_t e = configure_once(&cus)) return e;
    const int64_t big_tiles = b.first_tile[b.jobs];
    const int force = knob(SAMO_KNOB_WGRAD_TILE, 0);           // tuning and test aid: 128 or 256
    const int round = knob(SAMO_KNOB_WGRAD_ROUND, 0);          // test aid: tiles per round in place of the CU count
    if (round > 0) cus = round;
    // Large tiles in whole rounds of the compute units; what is left over after the last whole
    // round goes to the small shape when that is the quicker way to finish it: up to half a round
    // of large tiles is at most two rounds of small ones, and a small round takes 0.4 of a large.
    int64_t as_big = big_tiles, as_small = 0;
    if (force == kSmallTile) as_big = 0, as_small = big_tiles;
    else if (force != kBigTile && cus > 0 && big_tiles % cus != 0 && big_tiles % cus <= cus / 2) {
        as_small = big_tiles % cus;
        as_big = big_tiles - as_small;
    }
    auto launch = [&](bool small, unsigned blocks) {
        const unsigned grid = (blocks + 7) / 8 * 8;             // whole rounds of the 8 XCDs; the surplus exits at once
        if (small) {
            if (out_kind == kOutF32) wgrad_small_kernel<kOutF32><<<dim3(grid), dim3(kWgThreads), kLdsBytes, s>>>(b);
            else wgrad_small_kernel<kOutF16><<<dim3(grid), dim3(kWgThreads), kLdsBytes, s>>>(b);
        } else {
            if (out_kind == kOutF32) wgrad_big_kernel<kOutF32><<<dim3(grid), dim3(kWgThreads), kLdsBytes, s>>>(b);
            else wgrad_big_kernel<kOutF16><<<dim3(grid), dim3(kWgThreads), kLdsBytes, s>>>(b);
        }
    };
    if (as_big > 0) {
        b.quadrants = 0; b.first = 0; b.tiles = as_big;
        launch(false, (unsigned)as_big);
    }
    if (as_small > 0) {
        b.quadrants = 1; b.first = as_big; b.tiles = as_small;
        launch(true, (unsigned)(as_small * 4));
    }
    return hipGetLastError();
}

}  // namespace samo
