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
// original lists: it only needs to know where each block's slice starts.  Two more write the matrix in the
// paper's two other encodings (Sec. 3: inverted index, value compression) for the entry points that read those.
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

// Inverted index (Sec. 3 of the paper): the two ascending lists of a column merged into one, ascending in the row
// number, a -1 entry of row i stored as ~i.  Column n's merged list starts at col_start_pos[n] + col_start_neg[n].
// One thread per entry: its place in the merged list is its place in its own list plus the number of entries of the
// other list with a smaller row (no row is in both).  SIGN: the entries of the -1 list.
template <bool SIGN>
__global__ void __launch_bounds__(kThreads)
k_merge_signed(const int32_t *__restrict__ cs_own, const int32_t *__restrict__ cs_other,
               const int32_t *__restrict__ ri_own, const int32_t *__restrict__ ri_other, int32_t *__restrict__ merged,
               int N, int nnz_own)
{
    const int i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= nnz_own) return;
    // the column of entry i: the last n with cs_own[n] <= i
    int lo = 0, hi = N;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (cs_own[mid] <= i) lo = mid; else hi = mid;
    }
    const int n = lo, row = ri_own[i];
    const int smaller = lower_bound_dev(ri_other, cs_other[n], cs_other[n + 1], row) - cs_other[n];
    merged[cs_own[n] + cs_other[n] + (i - cs_own[n]) + smaller] = SIGN ? ~row : row;
}

// Value compression (Sec. 3 of the paper): five consecutive rows of a column as one base-3 number, digit 0 / 1 / 2 for
// an entry 0 / +1 / -1, first row most significant.  One thread per (chunk of 16 groups, column) reads the 80 rows
// from the row sets and stores its 16 bytes at once.
__global__ void __launch_bounds__(kThreads)
k_pack5(const unsigned long long *__restrict__ masks, uint8_t *__restrict__ packed, int n_pad, int n_kblocks,
        int n_chunks5)
{
    const long long id = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (id >= (long long)n_pad * n_chunks5) return;
    const int n = (int)(id % n_pad), chunk = (int)(id / n_pad);
    unsigned long long pos = 0, neg = 0;
    int have_kb = -1;
    uint32_t words[kChunk5 / 4];
#pragma unroll
    for (int j = 0; j < kChunk5; ++j) {
        unsigned code = 0;
#pragma unroll
        for (int r = 0; r < 5; ++r) {
            const long long row = ((long long)chunk * kChunk5 + j) * 5 + r;
            const int kb = (int)(row >> 6);
            unsigned digit = 0;
            if (kb < n_kblocks) {
                if (kb != have_kb) {
                    pos = masks[2 * ((size_t)kb * n_pad + n)];
                    neg = masks[2 * ((size_t)kb * n_pad + n) + 1];
                    have_kb = kb;
                }
                digit = (unsigned)((pos >> (row & 63)) & 1) + 2u * (unsigned)((neg >> (row & 63)) & 1);
            }
            code = code * 3 + digit;
        }
        if (j % 4 == 0) words[j / 4] = code; else words[j / 4] |= code << (8 * (j % 4));
    }
    uint4 v = {words[0], words[1], words[2], words[3]};
    *reinterpret_cast<uint4 *>(packed + (size_t)id * kChunk5) = v;
}

}  // namespace

hipError_t launch_reblock(const tcsc *t, hipStream_t stream)
{
    const tcsc_layout_t &l = t->layout;
    const DeviceTcsc d = device_view(t);
    hipError_t e = hipSuccess;
    if (l.forms & TCSC_FORM_ROWSETS) {
        const long long cells = (long long)l.n_pad * l.n_kblocks;
        const unsigned grid = (unsigned)((cells + kThreads - 1) / kThreads);
        hipLaunchKernelGGL(k_row_sets, dim3(grid), dim3(kThreads), 0, stream, d.col_start_pos, d.col_start_neg,
                           d.row_index_pos, d.row_index_neg, d.masks, l.N, l.n_pad, l.n_kblocks);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if (l.forms & TCSC_FORM_CUTS) {
        const long long cut_cells = (long long)l.n_pad * (l.n_cuts + 1);
        hipLaunchKernelGGL(k_list_cuts, dim3((unsigned)((cut_cells + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream,
                           d.col_start_pos, d.col_start_neg, d.row_index_pos, d.row_index_neg, d.list_cuts, l.N, l.n_pad,
                           l.n_cuts);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if ((l.forms & TCSC_FORM_SIGNED) && l.nnz_pos > 0)
        hipLaunchKernelGGL(k_merge_signed<false>, dim3((unsigned)((l.nnz_pos + kThreads - 1) / kThreads)), dim3(kThreads), 0,
                           stream, d.col_start_pos, d.col_start_neg, d.row_index_pos, d.row_index_neg, d.signed_index, l.N,
                           (int)l.nnz_pos);
    if ((l.forms & TCSC_FORM_SIGNED) && l.nnz_neg > 0)
        hipLaunchKernelGGL(k_merge_signed<true>, dim3((unsigned)((l.nnz_neg + kThreads - 1) / kThreads)), dim3(kThreads), 0,
                           stream, d.col_start_neg, d.col_start_pos, d.row_index_neg, d.row_index_pos, d.signed_index, l.N,
                           (int)l.nnz_neg);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (!(l.forms & TCSC_FORM_PACKED)) return hipSuccess;
    const long long pack_cells = (long long)l.n_pad * l.n_chunks5;
    hipLaunchKernelGGL(k_pack5, dim3((unsigned)((pack_cells + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream,
                       d.masks, d.packed, l.n_pad, l.n_kblocks, l.n_chunks5);
    return hipGetLastError();
}

}  // namespace tst
