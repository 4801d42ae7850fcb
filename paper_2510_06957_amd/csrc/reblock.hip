// GPU re-blocking pass: TCSC arrays (Sec. 2 of the paper) -> K-blocked per-column streams.
//
// The idea is the paper's BlockedTCSC (Sec. 3, "Blocking"): cut [0,K) into blocks so that the
// X entries one block touches fit in fast memory (here one LDS tile), and cut every column's
// +1 / -1 list at the block borders.  Because rows ascend inside a column, each piece is a
// contiguous slice of the original list, found by binary search.  The storage differs from the
// paper's: block-local row numbers, per-column streams, lists stored in 8-slot chunks so the
// kernel can fetch a chunk with one 32-byte scalar load (layout: tcsc_layout_t in tstgemm.h).
//
// Integer work only; three small kernels, run once per matrix at upload time.
#include "tstgemm_internal.h"

namespace tst {
namespace {

constexpr int kThreads = 256;

__device__ inline int lower_bound_dev(const int32_t *a, int lo, int hi, int key)
{
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (a[mid] < key) lo = mid + 1; else hi = mid;
    }
    return lo;
}

__device__ inline int pad_chunk_dev(int n) { return (n + kChunk - 1) & ~(kChunk - 1); }

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
        const int64_t lo = (int64_t)kb * kKBlock, hi = lo + kKBlock;
        const int klo = (int)lo, khi = hi > INT32_MAX ? INT32_MAX : (int)hi;
        const int p0 = csp[n], p1 = csp[n + 1], q0 = csn[n], q1 = csn[n + 1];
        const int a = lower_bound_dev(rip, p0, p1, klo);
        cp = (hi > INT32_MAX ? p1 : lower_bound_dev(rip, a, p1, khi)) - a;
        const int c = lower_bound_dev(rin, q0, q1, klo);
        cn = (hi > INT32_MAX ? q1 : lower_bound_dev(rin, c, q1, khi)) - c;
    }
    seg_count[id] = cp | (cn << 16);
}

// col_ptr[n + 1] = padded stream length of column n (turned into a running sum by k_scan)
__global__ void __launch_bounds__(kThreads)
k_col_len(const int32_t *__restrict__ seg_count, int64_t *__restrict__ col_ptr, int n_pad, int n_kblocks)
{
    const int n = blockIdx.x * kThreads + threadIdx.x;
    if (n >= n_pad) return;
    int64_t len = 0;
    for (int kb = 0; kb < n_kblocks; ++kb) {
        const int c = seg_count[(int64_t)kb * n_pad + n];
        len += pad_chunk_dev(c & 0xffff) + pad_chunk_dev((c >> 16) & 0xffff);
    }
    col_ptr[n + 1] = len;
    if (n == 0) col_ptr[0] = 0;
}

// In-place inclusive scan of col_ptr[1 .. n_pad] by one workgroup.
__global__ void __launch_bounds__(1024) k_scan(int64_t *__restrict__ col_ptr, int n_pad)
{
    __shared__ int64_t part[1024];
    const int t = threadIdx.x;
    const int per = (n_pad + 1023) / 1024;
    const int lo = t * per, hi = min(lo + per, n_pad);
    int64_t s = 0;
    for (int n = lo; n < hi; ++n) s += col_ptr[n + 1];
    part[t] = s;
    __syncthreads();
    for (int d = 1; d < 1024; d <<= 1) {
        const int64_t v = t >= d ? part[t - d] : 0;
        __syncthreads();
        part[t] += v;
        __syncthreads();
    }
    int64_t run = part[t] - s;   // sum of everything before this thread's slice
    for (int n = lo; n < hi; ++n) {
        run += col_ptr[n + 1];
        col_ptr[n + 1] = run;
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

// One thread per (column, K-block): copy the two list slices into the column's stream.
__global__ void __launch_bounds__(kThreads)
k_fill(const int32_t *__restrict__ csp, const int32_t *__restrict__ csn, const int32_t *__restrict__ rip,
       const int32_t *__restrict__ rin, const int32_t *__restrict__ seg_count, const int64_t *__restrict__ col_ptr,
       int32_t *__restrict__ stream, int N, int n_pad, int n_kblocks, int64_t stream_len)
{
    const int64_t id = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (id == 0)
        for (int i = 0; i < kChunk; ++i) stream[stream_len + i] = 0;   // slack behind the last chunk
    if (id >= (int64_t)n_pad * n_kblocks) return;
    const int n = (int)(id % n_pad), kb = (int)(id / n_pad);
    if (n >= N) return;
    int64_t off = col_ptr[n];
    int before_p = 0, before_n = 0;
    for (int j = 0; j < kb; ++j) {
        const int c = seg_count[(int64_t)j * n_pad + n];
        const int cp = c & 0xffff, cn = (c >> 16) & 0xffff;
        before_p += cp;
        before_n += cn;
        off += pad_chunk_dev(cp) + pad_chunk_dev(cn);
    }
    const int c = seg_count[(int64_t)kb * n_pad + n];
    const int cp = c & 0xffff, cn = (c >> 16) & 0xffff;
    const int base_row = kb * kKBlock;
    write_list(stream + off, rip + csp[n] + before_p, cp, base_row);
    write_list(stream + off + pad_chunk_dev(cp), rin + csn[n] + before_n, cn, base_row);
}

}  // namespace

hipError_t launch_reblock(const tcsc *t, hipStream_t stream)
{
    const tcsc_layout_t &l = t->layout;
    const DeviceTcsc d = device_view(t);
    const int64_t cells = (int64_t)l.n_pad * l.n_kblocks;
    const unsigned grid_cells = (unsigned)((cells + kThreads - 1) / kThreads);
    hipLaunchKernelGGL(k_count, dim3(grid_cells), dim3(kThreads), 0, stream, d.col_start_pos, d.col_start_neg,
                       d.row_index_pos, d.row_index_neg, d.seg_count, l.N, l.n_pad, l.n_kblocks);
    hipLaunchKernelGGL(k_col_len, dim3((l.n_pad + kThreads - 1) / kThreads), dim3(kThreads), 0, stream, d.seg_count,
                       d.col_ptr, l.n_pad, l.n_kblocks);
    hipLaunchKernelGGL(k_scan, dim3(1), dim3(1024), 0, stream, d.col_ptr, l.n_pad);
    hipLaunchKernelGGL(k_fill, dim3(grid_cells), dim3(kThreads), 0, stream, d.col_start_pos, d.col_start_neg,
                       d.row_index_pos, d.row_index_neg, d.seg_count, d.col_ptr, d.stream, l.N, l.n_pad, l.n_kblocks,
                       l.stream_len);
    return hipGetLastError();
}

}  // namespace tst
