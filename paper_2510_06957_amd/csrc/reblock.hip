// GPU re-blocking pass: TCSC arrays (Sec. 2 of the paper) -> K-blocked row sets.
//
// The idea is the paper's BlockedTCSC (Sec. 3, "Blocking"): cut [0,K) into blocks so that the
// X entries one block touches fit in fast memory (here one LDS tile), cut every column's
// +1 / -1 list at the block borders, and store the pieces block after block.  Because rows
// ascend inside a column, each piece is a contiguous slice of the original list, found by
// binary search.  The storage differs from the paper's: a block spans 64 rows, so a piece is
// kept as a 64-bit set of block-local row numbers instead of a list of 32-bit indices
// (layout: tcsc_layout_t in tstgemm.h).
//
// A second small kernel cuts the lists at multiples of 256 rows for the small-tile kernel, which walks the
// original lists: it only needs to know where each block's slice starts.
//
// Integer work only, run once per matrix at upload time.
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

// The rows of list rows[lo..hi) that fall into K-block kb, as a set of block-local row numbers.
__device__ inline unsigned long long row_set(const int32_t *rows, int lo, int hi, int kb)
{
    const long long k_lo = (long long)kb * kKBlock, k_hi = k_lo + kKBlock;
    unsigned long long set = 0;
    for (int i = lower_bound_dev(rows, lo, hi, (int)k_lo); i < hi && rows[i] < k_hi; ++i)
        set |= 1ull << (rows[i] - k_lo);
    return set;
}

// One thread per (K-block, column).
__global__ void __launch_bounds__(kThreads)
k_row_sets(const int32_t *__restrict__ csp, const int32_t *__restrict__ csn, const int32_t *__restrict__ rip,
           const int32_t *__restrict__ rin, unsigned long long *__restrict__ masks, int N, int n_pad, int n_kblocks)
{
    const long long id = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (id >= (long long)n_pad * n_kblocks) return;
    const int n = (int)(id % n_pad), kb = (int)(id / n_pad);
    unsigned long long pos = 0, neg = 0;
    if (n < N) {
        pos = row_set(rip, csp[n], csp[n + 1], kb);
        neg = row_set(rin, csn[n], csn[n + 1], kb);
    }
    masks[2 * id] = pos;
    masks[2 * id + 1] = neg;
}

// One thread per (cut, column): where the rows >= cut * kCutRows start in the column's two lists.
__global__ void __launch_bounds__(kThreads)
k_list_cuts(const int32_t *__restrict__ csp, const int32_t *__restrict__ csn, const int32_t *__restrict__ rip,
            const int32_t *__restrict__ rin, int32_t *__restrict__ cuts, int N, int n_pad, int n_cuts)
{
    const long long id = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (id >= (long long)n_pad * (n_cuts + 1)) return;
    const int n = (int)(id % n_pad), c = (int)(id / n_pad);
    int pos = 0, neg = 0;
    if (n < N) {
        const long long row = (long long)c * kCutRows;
        pos = c == n_cuts ? csp[n + 1] : lower_bound_dev(rip, csp[n], csp[n + 1], (int)row);
        neg = c == n_cuts ? csn[n + 1] : lower_bound_dev(rin, csn[n], csn[n + 1], (int)row);
    }
    cuts[2 * id] = pos;
    cuts[2 * id + 1] = neg;
}

}  // namespace

hipError_t launch_reblock(const tcsc *t, hipStream_t stream)
{
    const tcsc_layout_t &l = t->layout;
    const DeviceTcsc d = device_view(t);
    const long long cells = (long long)l.n_pad * l.n_kblocks;
    const unsigned grid = (unsigned)((cells + kThreads - 1) / kThreads);
    hipLaunchKernelGGL(k_row_sets, dim3(grid), dim3(kThreads), 0, stream, d.col_start_pos, d.col_start_neg,
                       d.row_index_pos, d.row_index_neg, d.masks, l.N, l.n_pad, l.n_kblocks);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const long long cut_cells = (long long)l.n_pad * (l.n_cuts + 1);
    hipLaunchKernelGGL(k_list_cuts, dim3((unsigned)((cut_cells + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream,
                       d.col_start_pos, d.col_start_neg, d.row_index_pos, d.row_index_neg, d.list_cuts, l.N, l.n_pad,
                       l.n_cuts);
    return hipGetLastError();
}

}  // namespace tst
