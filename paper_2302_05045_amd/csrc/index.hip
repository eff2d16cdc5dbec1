// Mask -> index construction (the paper's ind_i, Section III and III-B) for gfx950.
//
// The pruner's output arrives as a byte mask over the flattened layer.  The mask is read ONCE.
// A workgroup of eight wavefronts owns a block of 64, 128 or 256 consecutive segments of
// SAMO_SEG_ELEMS = 1024 mask bytes, taken in passes of 64; in a pass a wavefront takes eight of
// them, every lane loading 16 bytes of each, so a segment is one coalesced 1 KiB access and eight
// are in flight per lane.  The kept bytes are counted per lane (popcount of a 16-bit flag word)
// and scanned across the wave, which gives every lane its offset within the segment and the
// segment its total; the number of kept elements in front of the workgroup then comes from a
// chained scan across workgroups (each publishes its own count at once and the running total as
// soon as it knows it; a successor sums the counts back to the nearest running total); finally
// the ascending int32 positions are produced from the flag words still held in registers,
// collected per segment in LDS and stored as contiguous runs.  All integer work: one read of the
// mask plus the write of the index, about 100 vector-ALU instructions per segment and wave.
//
// The chain lives in seg_ptr itself: seg_ptr[e], e the end of a workgroup's block of segments, is
// the number of kept elements up to there — exactly the running total the next workgroup needs.
// While unknown it holds kEmpty, then -1 - (own count), then the final value.  Workgroups take
// their blocks in the order of a ticket drawn at start, so every predecessor of a running
// workgroup is itself running or done and the wait for it ends; the wait is bounded all the same,
// and a workgroup that gives up marks its block kPoison, which its successors pass on and the
// last block of the job reports as *nnz = -1.
#include "common.h"

namespace samo {
namespace {

constexpr int kIndexThreads = 512;        // index_kernel: eight wavefronts per workgroup
constexpr int kWavesPerWg = kIndexThreads / 64;

// bit (8*b + 7) set for every non-zero byte b of x
__device__ __forceinline__ uint32_t nonzero_byte_flags(uint32_t x)
{
    return (((x & 0x7f7f7f7fu) + 0x7f7f7f7fu) | x) & 0x80808080u;
}

// 16-bit flag word for the 16 mask bytes owned by this lane; bytes at or beyond n read as 0.
__device__ __forceinline__ uint32_t lane_flags(const uint8_t *__restrict__ mask, int64_t n, int64_t first)
{
    uint32_t w[4] = {0u, 0u, 0u, 0u};
    if (first + 16 <= n) {
        typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
        const u32x4 q = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(mask + first));   // read once
        w[0] = q.x; w[1] = q.y; w[2] = q.z; w[3] = q.w;
    } else {
        for (int b = 0; b < 16; ++b)
            if (first + b < n) w[b >> 2] |= (uint32_t)mask[first + b] << (8 * (b & 3));
    }
    // Every non-zero byte is now 0x80: a dot product of the four bytes of a word with the weights
    // 1, 2, 4, 8 (16 .. 128 for the next word, accumulated) is 128 times their flag bits in order.
    uint32_t lo = __builtin_amdgcn_udot4(nonzero_byte_flags(w[0]), 0x08040201u, 0u, false);
    lo = __builtin_amdgcn_udot4(nonzero_byte_flags(w[1]), 0x80402010u, lo, false);
    uint32_t hi = __builtin_amdgcn_udot4(nonzero_byte_flags(w[2]), 0x08040201u, 0u, false);
    hi = __builtin_amdgcn_udot4(nonzero_byte_flags(w[3]), 0x80402010u, hi, false);
    return (lo >> 7) | (hi << 1);
}

__device__ __forceinline__ int wave_sum(int x)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d, 64);
    return x;
}

// Inclusive scan over the 64 lanes with data-parallel primitives: a shifted add within each row of
// 16 lanes (four steps), then lane 15 of a row added to the whole next row and lane 31 to the upper
// half — the operands move inside the vector ALU, no trip through the LDS crossbar.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_add(int x)
{
    // lanes the pattern does not feed read 0 (bound_ctrl); rows outside ROW_MASK add 0
    return x + __builtin_amdgcn_update_dpp(0, x, CTRL, ROW_MASK, 0xf, true);
}

__device__ __forceinline__ int wave_inclusive_scan(int x, int lane)
{
    (void)lane;
    x = dpp_add<0x111, 0xf>(x);               // row_shr:1
    x = dpp_add<0x112, 0xf>(x);               // row_shr:2
    x = dpp_add<0x114, 0xf>(x);               // row_shr:4
    x = dpp_add<0x118, 0xf>(x);               // row_shr:8
    x = dpp_add<0x142, 0xa>(x);               // row_bcast:15 into rows 1 and 3
    x = dpp_add<0x143, 0xc>(x);               // row_bcast:31 into rows 2 and 3
    return x;
}

// Workgroup -> job lookup for the batched launches: the job table travels in the kernel
// argument segment (scalar loads, no device table to allocate or copy), wg_start is the
// exclusive prefix of the jobs' workgroup counts.
__device__ __forceinline__ int find_job(const IndexBatch &batch, int wg)
{
    int lo = 0, hi = batch.num;                 // invariant: wg_start[lo] <= wg < wg_start[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (batch.wg_start[mid] <= wg) lo = mid; else hi = mid;
    }
    return lo;
}

// A workgroup takes its block in PASSES passes of 64 KiB: in a pass every wave loads eight
// consecutive segments — all eight 16-byte loads of a lane in flight before anything is reduced —
// and keeps only their flag words (two to a register) for the fill.  The per-lane counts travel
// through the wave scans packed two to a register: a count is at most 1024, a 16-bit field is
// enough.  What a workgroup pays once whatever its block's size — drawing the ticket, waiting for
// its predecessors in the chain — is a dozen microseconds, against less than two for a pass, so a
// launch with enough mask to keep the compute units busy takes four passes per workgroup (256 KiB
// blocks), smaller ones two or one.
constexpr int kSegsPerPass = 8;           // per wave
constexpr int kMaxPasses = 4;
__host__ __device__ constexpr int segs_per_wg(int passes) { return kSegsPerPass * kWavesPerWg * passes; }

// States of a chain entry other than a final running total (which is >= 0).
constexpr int kEmpty = INT32_MIN;         // nothing published yet
constexpr int kPoison = INT32_MIN + 1;    // a predecessor gave up
__device__ __forceinline__ int encode_count(int c) { return -1 - c; }
__device__ __forceinline__ int decode_count(int v) { return -1 - v; }

__device__ __forceinline__ int chain_load(const int32_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void chain_store(int32_t *p, int v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// seg_ptr position of the chain entry of block b (blocks of `block_segs` segments): the end of its segments.
__device__ __forceinline__ int64_t chain_slot(int64_t b, int64_t nseg, int block_segs)
{
    const int64_t e = (b + 1) * block_segs;
    return e < nseg ? e : nseg;
}

// Prepares a batch: every job's seg_ptr[0] = 0 and *nnz = 0 (the ticket counter is one of these),
// every block's chain entry = kEmpty.
__global__ void __launch_bounds__(kThreads)
index_init_kernel(const IndexBatch batch)
{
    const int t = blockIdx.x * kThreads + threadIdx.x;
    if (t < batch.num) {
        batch.seg_ptr[t][0] = 0;
        *batch.nnz[t] = 0;
    }
    if (t < batch.wg_start[batch.num]) {
        const int job = find_job(batch, t);
        const int64_t nseg = (batch.n[job] + kSeg - 1) / kSeg;
        batch.seg_ptr[job][chain_slot(t - batch.wg_start[job], nseg, segs_per_wg(batch.passes))] = kEmpty;
    }
}

// Number of kept elements in front of block `blk` of a job (wave 0 of the workgroup, all lanes):
// sums the published counts of the predecessors back to the nearest running total, 64 chain
// entries per look (more per look did not pay: measured).  Returns kPoison if a predecessor gave
// up or never shows.
__device__ __forceinline__ int kept_before_block(const int32_t *seg_ptr, int64_t nseg, int block_segs, int blk, int lane,
                                                 int spin_limit)
{
    int prefix = 0;
    int back = blk - 1;                       // nearest predecessor not yet accounted for
    int spins = 0;
    while (back >= 0) {
        const int b = back - lane;            // lane i looks at block back - i
        int v = kEmpty;
        if (b >= 0) v = chain_load(seg_ptr + chain_slot(b, nseg, block_segs));
        const unsigned long long m_total = __ballot(b >= 0 && v >= 0);
        const int first_total = m_total ? __ffsll((long long)m_total) - 1 : 64;
        // the lanes in front of the first running total must all hold counts
        const bool wanted = lane <= first_total && b >= 0;
        if (__any(wanted && v == kPoison)) return kPoison;
        if (__any(wanted && v == kEmpty)) {
            if (++spins > spin_limit) return kPoison;
            __builtin_amdgcn_s_sleep(2);
            continue;
        }
        int part = 0;
        if (wanted) part = (lane == first_total) ? v : decode_count(v);
        prefix += wave_sum(part);
        if (first_total < 64) break;
        back -= 64;
    }
    return prefix;
}

template <int PASSES>
__global__ void __launch_bounds__(kIndexThreads)
index_kernel(const IndexBatch batch, int fill)
{
    constexpr int kSegsPerWave = kSegsPerPass * PASSES;
    constexpr int kSegsPerWg = segs_per_wg(PASSES);
    constexpr int kPerLane = kSegsPerWg / 64;     // segment counts a lane of wave 0 takes in the block's scan
    __shared__ int sh_ticket;
    __shared__ int sh_seg[kSegsPerWg];        // kept elements per segment, then in front of it within the block
    __shared__ int sh_base;                   // kept elements in front of the block, or kPoison
    __shared__ int32_t sh_stage[kWavesPerWg][kSeg];   // positions of one segment per wave, on their way out
    if (threadIdx.x == 0) sh_ticket = (int)atomicAdd(reinterpret_cast<unsigned long long *>(batch.ticket), 1ull);
    __syncthreads();
    const int ticket = sh_ticket;
    const int job = find_job(batch, ticket);
    const int blk = ticket - batch.wg_start[job];
    const int64_t n = batch.n[job];
    const int64_t nseg = (n + kSeg - 1) / kSeg;
    int32_t *__restrict__ seg_ptr = batch.seg_ptr[job];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t seg0 = ((int64_t)blk * kWavesPerWg + wave) * kSegsPerWave;     // segments beyond nseg read as empty

    uint32_t fp[PASSES][kSegsPerPass / 2];    // flag words of segments 2j (low half) and 2j + 1 (high half) of a pass
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        uint32_t f[kSegsPerPass];
#pragma unroll
        for (int q = 0; q < kSegsPerPass; ++q)
            f[q] = lane_flags(batch.mask[job], n, (seg0 + p * kSegsPerPass + q) * kSeg + lane * 16);
#pragma unroll
        for (int j = 0; j < kSegsPerPass / 2; ++j) {
            const int incl = wave_inclusive_scan(__popc(f[2 * j]) | (__popc(f[2 * j + 1]) << 16), lane);
            if (lane == 63) {                  // the last lane's inclusive prefixes are the segment totals
                int *dst = sh_seg + wave * kSegsPerWave + p * kSegsPerPass + 2 * j;
                dst[0] = incl & 0xffff;
                dst[1] = incl >> 16;
            }
            fp[p][j] = f[2 * j] | (f[2 * j + 1] << 16);
        }
        asm volatile("" ::: "memory");        // the next pass's loads are requested after this pass's flag words exist
    }
    __syncthreads();

    const int64_t slot = chain_slot(blk, nseg, kSegsPerWg);
    const bool last_block = (blk + 1 == batch.wg_start[job + 1] - batch.wg_start[job]);
    if (wave == 0) {
        int c[kPerLane], mine = 0;
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) {
            c[i] = sh_seg[kPerLane * lane + i];
            mine += c[i];
        }
        const int incl = wave_inclusive_scan(mine, lane);
        const int total = __shfl(incl, 63, 64);
        if (blk > 0 && lane == 0) chain_store(seg_ptr + slot, encode_count(total));
        const int before = kept_before_block(seg_ptr, nseg, kSegsPerWg, blk, lane, batch.spin_limit);
        if (lane == 0) {
            chain_store(seg_ptr + slot, before == kPoison ? kPoison : before + total);
            sh_base = before;
            if (last_block) *batch.nnz[job] = (before == kPoison) ? -1 : (int64_t)before + total;
        }
        int run = incl - mine;
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) {
            sh_seg[kPerLane * lane + i] = run;
            run += c[i];
        }
    }
    __syncthreads();
    const int base = sh_base;
    if (base == kPoison) return;

    // seg_ptr entries strictly inside the block (its first is the predecessor's chain entry)
    const int64_t first_seg = (int64_t)blk * kSegsPerWg;
    for (int t = threadIdx.x; t < kSegsPerWg; t += kIndexThreads)
        if (t >= 1 && first_seg + t < slot) seg_ptr[first_seg + t] = base + sh_seg[t];

    const int64_t cap = batch.cap[job];
    if (!fill || cap <= 0 || seg0 >= nseg) return;
    int32_t *__restrict__ idx = batch.idx[job];
    int32_t *stage = sh_stage[wave];           // this wave's own staging area: no workgroup barrier needed
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
#pragma unroll
        for (int j = 0; j < kSegsPerPass / 2; ++j) {
            const uint32_t pair[2] = {fp[p][j] & 0xffffu, fp[p][j] >> 16};
            const int cnt = __popc(pair[0]) | (__popc(pair[1]) << 16);
            const int incl = wave_inclusive_scan(cnt, lane);          // formed again: cheaper than keeping it
            const int ex = incl - cnt, tt = __builtin_amdgcn_readlane(incl, 63);
            const int excl[2] = {ex & 0xffff, ex >> 16}, tot[2] = {tt & 0xffff, tt >> 16};
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                // the segment's positions go to LDS in order, then leave as contiguous 256-byte stores
                const int sq = p * kSegsPerPass + 2 * j + h;
                const int first = (int)((seg0 + sq) * kSeg) + lane * 16;     // a layer's flat size fits int32
                int at = excl[h];
                uint32_t bits = pair[h];
                while (bits) {
                    const int b = __ffs(bits) - 1;
                    bits &= bits - 1;
                    stage[at++] = first + b;
                }
                __builtin_amdgcn_wave_barrier();
                const int64_t out0 = (int64_t)base + sh_seg[wave * kSegsPerWave + sq];
                for (int o = lane; o < tot[h]; o += 64)
                    if (out0 + o < cap) idx[out0 + o] = stage[o];
                __builtin_amdgcn_wave_barrier();
            }
        }
    }
}

__global__ void __launch_bounds__(kThreads)
seg_ptr_from_idx_kernel(const int32_t *__restrict__ idx, int64_t nnz, int64_t nseg, int32_t *__restrict__ seg_ptr)
{
    const int64_t s = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (s > nseg) return;
    const int64_t key = s * kSeg;          // first i with idx[i] >= key
    int64_t lo = 0, hi = nnz;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if ((int64_t)idx[mid] < key) lo = mid + 1; else hi = mid;
    }
    seg_ptr[s] = (int32_t)lo;
}

__global__ void set_flag_kernel(int32_t *flag, int32_t value) { *flag = value; }

__global__ void __launch_bounds__(kThreads)
validate_kernel(const int32_t *__restrict__ idx, int64_t nnz, int64_t n, int64_t nseg,
                const int32_t *__restrict__ seg_ptr, int32_t *__restrict__ ok)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    bool bad = false;
    if (i < nnz) {
        const int64_t j = idx[i];
        if (j < 0 || j >= n) bad = true;
        else if (i > 0 && (int64_t)idx[i - 1] >= j) bad = true;
        else if (seg_ptr) {
            const int64_t s = j / kSeg;
            if (!((int64_t)seg_ptr[s] <= i && i < (int64_t)seg_ptr[s + 1])) bad = true;
        }
    }
    if (seg_ptr && i <= nseg) {
        if (i == 0 && seg_ptr[0] != 0) bad = true;
        if (i == nseg && (int64_t)seg_ptr[nseg] != nnz) bad = true;
        if (i < nseg && seg_ptr[i] > seg_ptr[i + 1]) bad = true;
    }
    if (bad) *ok = 0;
}

}  // namespace

hipError_t launch_index_batch(const IndexBatch &batch, bool fill, hipStream_t s)
{
    if (batch.num <= 0) return hipSuccess;
    const int wgs = batch.wg_start[batch.num];
    const int init_threads = wgs > batch.num ? wgs : batch.num;
    index_init_kernel<<<dim3((unsigned)ceil_div(init_threads, kThreads)), dim3(kThreads), 0, s>>>(batch);
    if (wgs > 0) {
        const dim3 grid((unsigned)wgs), block(kIndexThreads);
        if (batch.passes == 4) index_kernel<4><<<grid, block, 0, s>>>(batch, fill ? 1 : 0);
        else if (batch.passes == 2) index_kernel<2><<<grid, block, 0, s>>>(batch, fill ? 1 : 0);
        else index_kernel<1><<<grid, block, 0, s>>>(batch, fill ? 1 : 0);
    }
    return hipGetLastError();
}

int64_t index_job_workgroups(int64_t n, int passes) { return ceil_div(ceil_div(n, kSeg), segs_per_wg(passes)); }

// Passes per workgroup for a launch over `mask_bytes` bytes of mask: the most for which the launch
// still has four rounds of workgroups (three of them fit a compute unit at a time).
int index_passes_for(int64_t mask_bytes, int compute_units)
{
    const int64_t wanted = (int64_t)compute_units * 3 * 4;
    for (int passes = kMaxPasses; passes > 1; passes /= 2)
        if (mask_bytes / ((int64_t)segs_per_wg(passes) * kSeg) >= wanted) return passes;
    return 1;
}

hipError_t launch_seg_ptr_from_idx(const int32_t *idx, int64_t nnz, int64_t n, int32_t *seg_ptr, hipStream_t s)
{
    const int64_t nseg = ceil_div(n, kSeg);
    seg_ptr_from_idx_kernel<<<dim3((unsigned)ceil_div(nseg + 1, kThreads)), dim3(kThreads), 0, s>>>(idx, nnz, nseg,
                                                                                                   seg_ptr);
    return hipGetLastError();
}

hipError_t launch_validate(const int32_t *idx, int64_t nnz, int64_t n, const int32_t *seg_ptr, int32_t *ok,
                           hipStream_t s)
{
    const int64_t nseg = ceil_div(n, kSeg);
    set_flag_kernel<<<dim3(1), dim3(1), 0, s>>>(ok, 1);
    const int64_t work = nnz > nseg + 1 ? nnz : nseg + 1;
    validate_kernel<<<dim3((unsigned)ceil_div(work, kThreads)), dim3(kThreads), 0, s>>>(idx, nnz, n, nseg, seg_ptr,
                                                                                       ok);
    return hipGetLastError();
}

}  // namespace samo
