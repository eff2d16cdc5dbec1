// Mask -> index construction (the paper's ind_i, Section III and III-B) for gfx950.
//
// The pruner's output arrives as a byte mask over the flattened layer.  One
// 64-lane wavefront owns one segment of SAMO_SEG_ELEMS = 1024 mask bytes: every
// lane loads 16 bytes, so a wave reads its segment with one coalesced 1 KiB
// access.  Pass 1 counts the kept bytes per segment, a single-workgroup scan
// turns the counts into seg_ptr (exclusive prefix), pass 2 re-reads the mask and
// writes the ascending int32 positions using a wave-level exclusive scan of the
// lanes' counts.  All integer work; bound by the two mask reads.
#include "common.h"

namespace samo {
namespace {

constexpr int kWavesPerWg = kThreads / 64;
constexpr int kScanThreads = 1024;

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
        const uint4 q = *reinterpret_cast<const uint4 *>(mask + first);
        w[0] = q.x; w[1] = q.y; w[2] = q.z; w[3] = q.w;
    } else {
        for (int b = 0; b < 16; ++b)
            if (first + b < n) w[b >> 2] |= (uint32_t)mask[first + b] << (8 * (b & 3));
    }
    uint32_t f = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t t = nonzero_byte_flags(w[q]) >> 7;   // bits 0, 8, 16, 24
        f |= ((t & 1u) | ((t >> 7) & 2u) | ((t >> 14) & 4u) | ((t >> 21) & 8u)) << (4 * q);
    }
    return f;
}

__device__ __forceinline__ int wave_sum(int x)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d, 64);
    return x;
}

__device__ __forceinline__ int wave_inclusive_scan(int x, int lane)
{
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int y = __shfl_up(x, d, 64);
        if (lane >= d) x += y;
    }
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

// A wave takes kSegsPerWave consecutive segments: four independent 16-byte loads per lane are in
// flight before anything is reduced, and the four per-lane counts travel through the wave
// reduction (or scan) packed two to a register — a count is at most 1024, a 16-bit field is enough.
constexpr int kSegsPerWave = 4;
constexpr int kSegsPerWg = kSegsPerWave * kWavesPerWg;

__global__ void __launch_bounds__(kThreads)
count_kernel(const IndexBatch batch)
{
    const int job = find_job(batch, blockIdx.x);
    const int64_t n = batch.n[job];
    const int64_t nseg = (n + kSeg - 1) / kSeg;
    const int lane = threadIdx.x & 63;
    const int64_t seg0 = ((int64_t)(blockIdx.x - batch.wg_start[job]) * kWavesPerWg + (threadIdx.x >> 6)) * kSegsPerWave;
    if (seg0 >= nseg) return;
    uint32_t f[kSegsPerWave];
#pragma unroll
    for (int q = 0; q < kSegsPerWave; ++q) f[q] = lane_flags(batch.mask[job], n, (seg0 + q) * kSeg + lane * 16);
    const int lo = wave_sum(__popc(f[0]) | (__popc(f[1]) << 16));
    const int hi = wave_sum(__popc(f[2]) | (__popc(f[3]) << 16));
    if (lane < kSegsPerWave && seg0 + lane < nseg) {
        const int packed = (lane < 2) ? lo : hi;
        batch.seg_ptr[job][seg0 + lane] = (lane & 1) ? (packed >> 16) : (packed & 0xffff);
    }
}

// In-place exclusive scan of a job's seg_ptr[0 .. nseg] where the last entry counts as 0 on
// input, so that seg_ptr[nseg] receives the grand total; the total is also stored to *nnz.
// One workgroup per job: every thread owns a contiguous run of ceil(len / 1024) entries (summed
// and rewritten serially), and one block-wide scan of the 1024 run totals links the runs.
__global__ void __launch_bounds__(kScanThreads)
scan_kernel(const IndexBatch batch)
{
    __shared__ int wave_tot[kScanThreads / 64];
    const int job = blockIdx.x;
    int32_t *__restrict__ a = batch.seg_ptr[job];
    const int64_t len = (batch.n[job] + kSeg - 1) / kSeg + 1;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t per = (len + kScanThreads - 1) / kScanThreads;
    const int64_t lo = (int64_t)tid * per;
    const int64_t hi = (lo + per < len) ? lo + per : len;
    int sum = 0;
    for (int64_t i = lo; i < hi; ++i) sum += (i < len - 1) ? a[i] : 0;
    const int incl = wave_inclusive_scan(sum, lane);
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    if (wave == 0) {
        const int t = (lane < kScanThreads / 64) ? wave_tot[lane] : 0;
        const int ti = wave_inclusive_scan(t, lane);
        if (lane < kScanThreads / 64) wave_tot[lane] = ti - t;     // exclusive prefix of the waves
        if (lane == kScanThreads / 64 - 1) *batch.nnz[job] = (int64_t)ti;   // grand total
    }
    __syncthreads();
    int run = wave_tot[wave] + incl - sum;                          // exclusive prefix of this thread's run
    for (int64_t i = lo; i < hi; ++i) {
        const int x = (i < len - 1) ? a[i] : 0;
        a[i] = run;
        run += x;
    }
}

__global__ void __launch_bounds__(kThreads)
fill_kernel(const IndexBatch batch)
{
    const int job = find_job(batch, blockIdx.x);
    const int64_t n = batch.n[job];
    const int64_t cap = batch.cap[job];
    const int64_t nseg = (n + kSeg - 1) / kSeg;
    const int lane = threadIdx.x & 63;
    const int64_t seg0 = ((int64_t)(blockIdx.x - batch.wg_start[job]) * kWavesPerWg + (threadIdx.x >> 6)) * kSegsPerWave;
    if (seg0 >= nseg || cap <= 0) return;
    int32_t *__restrict__ idx = batch.idx[job];
    uint32_t f[kSegsPerWave];
    int base[kSegsPerWave];
#pragma unroll
    for (int q = 0; q < kSegsPerWave; ++q) {
        f[q] = lane_flags(batch.mask[job], n, (seg0 + q) * kSeg + lane * 16);
        base[q] = (seg0 + q < nseg) ? batch.seg_ptr[job][seg0 + q] : 0;
    }
    const int c01 = __popc(f[0]) | (__popc(f[1]) << 16);
    const int c23 = __popc(f[2]) | (__popc(f[3]) << 16);
    const int e01 = wave_inclusive_scan(c01, lane) - c01;       // exclusive lane prefixes, two per register
    const int e23 = wave_inclusive_scan(c23, lane) - c23;
    const int excl[kSegsPerWave] = {e01 & 0xffff, e01 >> 16, e23 & 0xffff, e23 >> 16};
#pragma unroll
    for (int q = 0; q < kSegsPerWave; ++q) {
        const int64_t first = (seg0 + q) * kSeg + lane * 16;
        int64_t out = (int64_t)base[q] + excl[q];
        uint32_t bits = f[q];
        while (bits) {
            const int b = __ffs(bits) - 1;
            bits &= bits - 1;
            if (out < cap) idx[out] = (int32_t)(first + b);
            ++out;
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
    const int wgs = batch.wg_start[batch.num];
    if (batch.num <= 0) return hipSuccess;
    if (wgs > 0) count_kernel<<<dim3((unsigned)wgs), dim3(kThreads), 0, s>>>(batch);
    scan_kernel<<<dim3((unsigned)batch.num), dim3(kScanThreads), 0, s>>>(batch);
    if (fill && wgs > 0) fill_kernel<<<dim3((unsigned)wgs), dim3(kThreads), 0, s>>>(batch);
    return hipGetLastError();
}

int64_t index_job_workgroups(int64_t n) { return ceil_div(ceil_div(n, kSeg), kSegsPerWg); }

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
