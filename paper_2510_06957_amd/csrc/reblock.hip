// GPU re-blocking pass: TCSC arrays (Sec. 2 of the paper) -> K-blocked index streams.
//
// The idea is the paper's BlockedTCSC (Sec. 3, "Blocking"): cut [0,K) into blocks so that the
// X entries one block touches fit in fast memory (here one LDS tile), cut every column's
// +1 / -1 list at the block borders, and store the pieces block after block.  Because rows
// ascend inside a column, each piece is a contiguous slice of the original list, found by
// binary search.  The storage differs from the paper's: block-local row numbers, and lists
// stored in 8-slot chunks so that the kernel can fetch a chunk with one 32-byte scalar load
// (layout: tcsc_layout_t in tstgemm.h).
//
// Integer work only; a handful of small kernels, run once per matrix at upload time.
#include "tstgemm_internal.h"

namespace tst {
namespace {

constexpr int kThreads = 256;
constexpr int kScanItems = 4;                       // cells per thread in the block scans
constexpr int kScanTile = kThreads * kScanItems;    // cells per workgroup in the block scans

__device__ inline int lower_bound_dev(const int32_t *a, int lo, int hi, int key)
{
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (a[mid] < key) lo = mid + 1; else hi = mid;
    }
    return lo;
}

__device__ inline unsigned chunks_of(int n) { return (unsigned)(n + kChunk - 1) / kChunk; }
__device__ inline unsigned cell_chunks(int c) { return chunks_of(c & 0xffff) + chunks_of((c >> 16) & 0xffff); }

// First entry of column n's list `rows[lo..hi)` that is >= the first row of K-block kb, and the number of
// entries inside the block.
__device__ inline void slice_of(const int32_t *rows, int lo, int hi, int kb, int &first, int &count)
{
    const int64_t k_lo = (int64_t)kb * kKBlock, k_hi = k_lo + kKBlock;
    first = lower_bound_dev(rows, lo, hi, (int)k_lo);
    const int last = k_hi > INT32_MAX ? hi : lower_bound_dev(rows, first, hi, (int)k_hi);
    count = last - first;
}

// seg_count[kb][n] = (#+1 rows of column n in K-block kb) | (#-1 rows) << 16
__global__ void __launch_bounds__(kThreads)
k_count(const int32_t *__restrict__ csp, const int32_t *__restrict__ csn, const int32_t *__restrict__ rip,
        const int32_t *__restrict__ rin, int32_t *__restrict__ seg_count, int N, int n_pad, int n_kblocks)
{
    const int64_t id = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (id >= (int64_t)n_pad * n_kblocks) return;
    const int n = (int)(id % n_pad), kb = (int)(id / n_pad);
    int cp = 0, cn = 0;
    if (n < N) {
        int first;
        slice_of(rip, csp[n], csp[n + 1], kb, first, cp);
        slice_of(rin, csn[n], csn[n + 1], kb, first, cn);
    }
    seg_count[id] = cp | (cn << 16);
}

// Exclusive scan of the cells' chunk counts in storage order (kb-major), three steps:
// per-tile totals, scan of the totals by one workgroup, per-tile scan with the tile's offset.
__global__ void __launch_bounds__(kThreads)
k_tile_sums(const int32_t *__restrict__ seg_count, unsigned long long *__restrict__ tile_sum, int64_t cells)
{
    __shared__ unsigned long long part[kThreads];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
    unsigned long long s = 0;
    for (int i = 0; i < kScanItems; ++i)
        if (base + i < cells) s += cell_chunks(seg_count[base + i]);
    part[threadIdx.x] = s;
    __syncthreads();
    for (int d = kThreads / 2; d > 0; d >>= 1) {
        if ((int)threadIdx.x < d) part[threadIdx.x] += part[threadIdx.x + d];
        __syncthreads();
    }
    if (threadIdx.x == 0) tile_sum[blockIdx.x] = part[0];
}

__global__ void __launch_bounds__(1024) k_scan_tiles(unsigned long long *__restrict__ tile_sum, int n_tiles)
{
    __shared__ unsigned long long part[1024];
    const int t = threadIdx.x;
    const int per = (n_tiles + 1023) / 1024;
    const int lo = min(t * per, n_tiles), hi = min(lo + per, n_tiles);
    unsigned long long s = 0;
    for (int i = lo; i < hi; ++i) s += tile_sum[i];
    part[t] = s;
    __syncthreads();
    for (int d = 1; d < 1024; d <<= 1) {
        const unsigned long long v = t >= d ? part[t - d] : 0;
        __syncthreads();
        part[t] += v;
        __syncthreads();
    }
    unsigned long long run = part[t] - s;   // everything before this thread's slice
    for (int i = lo; i < hi; ++i) {
        const unsigned long long v = tile_sum[i];
        tile_sum[i] = run;                  // exclusive
        run += v;
    }
}

__global__ void __launch_bounds__(kThreads)
k_seg_ptr(const int32_t *__restrict__ seg_count, const unsigned long long *__restrict__ tile_sum,
          uint32_t *__restrict__ seg_ptr, int64_t cells)
{
    __shared__ unsigned long long part[kThreads];
    const int t = threadIdx.x;
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)t * kScanItems;
    unsigned v[kScanItems];
    unsigned long long s = 0;
    for (int i = 0; i < kScanItems; ++i) {
        v[i] = base + i < cells ? cell_chunks(seg_count[base + i]) : 0u;
        s += v[i];
    }
    part[t] = s;
    __syncthreads();
    for (int d = 1; d < kThreads; d <<= 1) {
        const unsigned long long u = t >= d ? part[t - d] : 0;
        __syncthreads();
        part[t] += u;
        __syncthreads();
    }
    unsigned long long run = tile_sum[blockIdx.x] + part[t] - s;
    for (int i = 0; i < kScanItems; ++i) {
        if (base + i < cells) seg_ptr[base + i] = (uint32_t)run;
        run += v[i];
    }
}

// Slot of entry e (0 <= e < r) inside a partial chunk holding r < 8 entries.
__device__ inline int tail_slot(int e, int r)
{
    const int four = r & 4, two = r & 2;
    if (e < four) return e;
    e -= four;
    if (e < two) return 4 + e;
    return 6;
}

__device__ inline void write_list(int32_t *__restrict__ dst, const int32_t *__restrict__ src, int count, int base_row)
{
    const int full = count & ~(kChunk - 1), r = count - full;
    for (int i = 0; i < full; ++i) dst[i] = src[i] - base_row;
    if (r) {
        for (int i = 0; i < kChunk; ++i) dst[full + i] = 0;
        for (int e = 0; e < r; ++e) dst[full + tail_slot(e, r)] = src[full + e] - base_row;
    }
}

// One thread per (K-block, column): copy the two list slices to their place in the stream.
__global__ void __launch_bounds__(kThreads)
k_fill(const int32_t *__restrict__ csp, const int32_t *__restrict__ csn, const int32_t *__restrict__ rip,
       const int32_t *__restrict__ rin, const uint32_t *__restrict__ seg_ptr, int32_t *__restrict__ stream, int N,
       int n_pad, int n_kblocks, int64_t stream_len)
{
    const int64_t id = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (id == 0)
        for (int i = 0; i < kStreamSlack; ++i) stream[stream_len + i] = 0;   // slack behind the last chunk
    if (id >= (int64_t)n_pad * n_kblocks) return;
    const int n = (int)(id % n_pad), kb = (int)(id / n_pad);
    if (n >= N) return;
    int first_p, cp, first_n, cn;
    slice_of(rip, csp[n], csp[n + 1], kb, first_p, cp);
    slice_of(rin, csn[n], csn[n + 1], kb, first_n, cn);
    int32_t *dst = stream + (int64_t)seg_ptr[id] * kChunk;
    const int base_row = kb * kKBlock;
    write_list(dst, rip + first_p, cp, base_row);
    write_list(dst + chunks_of(cp) * kChunk, rin + first_n, cn, base_row);
}

}  // namespace

hipError_t launch_reblock(const tcsc *t, hipStream_t stream)
{
    const tcsc_layout_t &l = t->layout;
    const DeviceTcsc d = device_view(t);
    const int64_t cells = (int64_t)l.n_pad * l.n_kblocks;
    const unsigned grid_cells = (unsigned)((cells + kThreads - 1) / kThreads);
    const int n_tiles = (int)((cells + kScanTile - 1) / kScanTile);
    // The tile totals live at the start of the partial-sum workspace: it is unused until the first tstgemm().
    if ((size_t)n_tiles * sizeof(unsigned long long) > kWorkspaceBytes - kCounterBytes) return hipErrorInvalidValue;
    unsigned long long *tile_sum = reinterpret_cast<unsigned long long *>(d.partials);
    hipLaunchKernelGGL(k_count, dim3(grid_cells), dim3(kThreads), 0, stream, d.col_start_pos, d.col_start_neg,
                       d.row_index_pos, d.row_index_neg, d.seg_count, l.N, l.n_pad, l.n_kblocks);
    hipLaunchKernelGGL(k_tile_sums, dim3(n_tiles), dim3(kThreads), 0, stream, d.seg_count, tile_sum, cells);
    hipLaunchKernelGGL(k_scan_tiles, dim3(1), dim3(1024), 0, stream, tile_sum, n_tiles);
    hipLaunchKernelGGL(k_seg_ptr, dim3(n_tiles), dim3(kThreads), 0, stream, d.seg_count, tile_sum, d.seg_ptr, cells);
    hipLaunchKernelGGL(k_fill, dim3(grid_cells), dim3(kThreads), 0, stream, d.col_start_pos, d.col_start_neg,
                       d.row_index_pos, d.row_index_neg, d.seg_ptr, d.stream, l.N, l.n_pad, l.n_kblocks, l.stream_len);
    return hipGetLastError();
}

}  // namespace tst
