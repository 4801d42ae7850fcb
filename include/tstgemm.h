/*
 * tstgemm -- sparse ternary GEMM  Y = X W + b  for one AMD MI355X (gfx950).
 *
 * C ABI of libtstgemm.so.  Plain pointers and sizes only; every pointer argument says
 * whether it is HOST or DEVICE memory.  All functions return 0 (TSTGEMM_OK) or a negative
 * TSTGEMM_E* code; tcsc_strerror() turns a code into text.  No function throws, aborts or
 * prints.  Besides what a handle owns the library keeps three pieces of global state: the tuning
 * overrides of tstgemm_set_tuning(), the choice of tstgemm_set_decode_lists() and the event pair of
 * tstgemm_profile_events().
 *
 * The operation is Eq. 1 of the paper (Sec. 2): X is dense fp32 (M x K, row-major), W is a
 * K x N matrix with entries in {-1, 0, +1}, b (N) is added to every row of the product,
 * Y is fp32 (M x N, row-major).  W is held in the TCSC format of Sec. 2: four int32 arrays,
 * col_start_pos / col_start_neg (N+1 column pointers) and row_index_pos / row_index_neg
 * (row numbers of the +1 / -1 entries, column after column, ascending inside a column; the
 * entries of column j are [col_start[j], col_start[j+1])).  The product is evaluated with
 * additions and subtractions only (BaseTCSC, Sec. 2): X entries whose weight is 0 are never
 * read, so a non-finite value there does not reach Y.
 */
#ifndef TSTGEMM_H
#define TSTGEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TSTGEMM_OK 0
#define TSTGEMM_EINVAL (-1)       /* null pointer, non-positive dimension, K/N differ from the handle's */
#define TSTGEMM_EFORMAT (-2)      /* W entry outside {-1,0,1}; pointers not monotone; row out of [0,K);
                                     rows of a column not strictly ascending; a row in both lists of a column */
#define TSTGEMM_ENOTUPLOADED (-3) /* tstgemm() on a handle that tcsc_upload() has not filled */
#define TSTGEMM_EHIP (-4)         /* a HIP runtime call failed (launch, copy) */
#define TSTGEMM_ENOMEM (-5)       /* host allocation failed, or the device buffer passed in is too small */
#define TSTGEMM_ETOOBIG (-6)      /* more than 2^31-1 entries in one sign list, or K >= 2^31 */

/* Opaque handle: owns a host copy of the four TCSC arrays; after tcsc_upload() it also
 * remembers (borrows, never frees) the caller's device buffer holding the device form. */
typedef struct tcsc tcsc_t;

/*
 * TCSC construction (Sec. 2, the four arrays), on the host.
 * W: HOST, K*N int8, row-major (W[k*N + n]), every value in {-1, 0, +1}.
 * *out receives a new handle (release with tcsc_destroy).  K, N >= 1.
 * Errors: EINVAL, EFORMAT (bad value), ETOOBIG, ENOMEM.
 */
int tcsc_build(const int8_t *W, int K, int N, tcsc_t **out);

/*
 * Handle from existing TCSC arrays (Sec. 2).  All four arrays HOST; they are validated
 * (see EFORMAT) and copied, the caller keeps ownership of its own.
 * col_start_*: N+1 entries, col_start[0] == 0; row_index_*: col_start_*[N] entries, 0-based.
 */
int tcsc_from_arrays(const int32_t *col_start_pos, const int32_t *col_start_neg,
                     const int32_t *row_index_pos, const int32_t *row_index_neg,
                     int K, int N, tcsc_t **out);

/* Dense form of the handle's matrix: W_out HOST, K*N int8 row-major, fully overwritten. */
int tcsc_to_dense(const tcsc_t *t, int8_t *W_out);

/* Shape and the number of +1 / -1 entries.  Any output pointer may be NULL. */
int tcsc_dims(const tcsc_t *t, int *K, int *N, int64_t *nnz_pos, int64_t *nnz_neg);

/* Borrow the handle's HOST copies of the four arrays (valid until tcsc_destroy). */
int tcsc_arrays(const tcsc_t *t, const int32_t **col_start_pos, const int32_t **col_start_neg,
                const int32_t **row_index_pos, const int32_t **row_index_neg);

/* Bytes of DEVICE memory tcsc_upload() needs for this matrix (256-byte aligned sections). */
int tcsc_device_bytes(const tcsc_t *t, size_t *bytes);

/*
 * Where things are inside the device buffer, byte offsets from its start.  The buffer holds
 * the four TCSC arrays unchanged (read by the small-M and small-tile kernels; each index array is
 * followed by 64 entries of slack, which those kernels may load but never use), their K-blocked
 * form (read by the large-M kernel) and the workspace of tstgemm().  K-blocking follows the idea
 * of BlockedTCSC (Sec. 3, "Blocking"): the rows [0,K) are cut into blocks of k_block = 64 rows
 * so that all X entries one block touches fit in the LDS, every column's two lists are cut at
 * the block borders, and the pieces are stored block after block.  A piece holds at most 64
 * distinct rows of one block, so it is stored as a 64-bit set: bit r of the word stands for
 * row kb*64 + r.  The kernel turns the set back into row numbers with find-first-set.
 *
 *   masks      uint64 [n_kblocks][n_pad][2]   [kb][n][0]: the +1 rows of column n inside K-block
 *                                             kb, [kb][n][1]: the -1 rows
 *   list_cuts  int32  [n_cuts + 1][n_pad][2]  for the small-tile kernel (M <= 64): the lists cut at multiples of
 *                                             cut_rows = 256 rows, as positions inside row_index_pos / _neg.
 *                                             [c][n][0]: index of the first entry of column n's +1 list whose row
 *                                             is >= c * 256 (c = n_cuts: the end of the list), [c][n][1]: the same
 *                                             for the -1 list.  Rows ascend inside a list, so the piece of a list
 *                                             inside a block of 256 rows is the slice between two cuts.
 *   col_start16_pos / _neg  int32 [N + 1]     only if K <= 65535 (has_lists16 != 0): the two lists of every column once
 *   row_index16_pos / _neg  uint16 [nnz16]    more, with 16-bit row numbers and every column's list padded to a multiple of
 *                                             8 entries (16 bytes) with the value K, which stands for a row of zeros;
 *                                             col_start16 are the pointers into these padded arrays.  Half the bytes for
 *                                             the small-M kernel, which is bound by them, and no partly used 16-byte piece.
 *   signed_index int32 [nnz_pos + nnz_neg]    the "inverted index" form (Sec. 3): the two lists of a column merged in
 *                                             ascending row order, +1 in row i stored as i, -1 as ~i; column n's
 *                                             entries are [col_start_pos[n] + col_start_neg[n],
 *                                             col_start_pos[n+1] + col_start_neg[n+1]); 64 entries of slack behind it.
 *                                             Read by tstgemm_signed().
 *   packed     uint8  [n_chunks5][n_pad][16]  the "value compression" form (Sec. 3): five consecutive rows of a
 *                                             column in one byte (see tcsc_packed_codes() for the code); group g
 *                                             of column n is byte [g / 16][n][g % 16], groups beyond ceil(K/5) and
 *                                             columns >= N hold code 0.  n_chunks5 = ceil(ceil(K/5) / 16).
 *                                             Read by tstgemm_packed().
 *   workspace  bytes  [workspace_bytes]       scratch of tstgemm(): split-K partial sums (32 MiB) and a tiled,
 *                                             transposed copy of (a slab of rows of) X (128 MiB, or one tile of
 *                                             256 rows over the padded K if that is larger)
 * n_pad = N rounded up to a multiple of 64; columns >= N have empty sets.
 */
typedef struct tcsc_layout {
    int32_t K, N, n_pad, k_block, n_kblocks, n_cuts;   /* n_cuts = K / 256 rounded up */
    int32_t n_chunks5, has_lists16;
    int64_t nnz_pos, nnz_neg;
    int64_t nnz16_pos, nnz16_neg;   /* entries of the padded 16-bit lists (0 without them) */
    size_t off_col_start_pos, off_col_start_neg, off_row_index_pos, off_row_index_neg;
    size_t off_masks, off_list_cuts;
    size_t off_col_start16_pos, off_col_start16_neg, off_row_index16_pos, off_row_index16_neg;
    size_t off_signed_index, off_packed, off_workspace, workspace_bytes, total_bytes;
} tcsc_layout_t;

int tcsc_layout(const tcsc_t *t, tcsc_layout_t *out);

/*
 * Copy the four arrays to the device and run the GPU re-blocking pass (row sets, list cuts, and the
 * two alternative encodings) into dev_buf.
 * dev_buf: DEVICE, at least tcsc_device_bytes() bytes, 256-byte aligned, owned by the
 * caller; the handle keeps the pointer until tcsc_destroy() and never frees it.  The buffer
 * must stay untouched while the handle is in use.  stream: a hipStream_t (NULL = the null
 * stream).  Work is enqueued on `stream`; the host arrays are read before the call returns.
 * Errors: EINVAL, ENOMEM (bytes too small), EHIP.
 */
int tcsc_upload(tcsc_t *t, void *dev_buf, size_t bytes, void *stream);

/*
 * Y = X W + b  (Eq. 1; evaluation as BaseTCSC, Sec. 2: gather-add the +1 rows, gather-subtract
 * the -1 rows, bias added once at the end).
 * X: DEVICE fp32 M*K row-major.  b: DEVICE fp32 N, or NULL for b = 0.  Y: DEVICE fp32 M*N
 * row-major, fully overwritten; must not overlap X, b or the handle's device buffer.
 * M >= 1 arbitrary; K, N must equal the handle's.  M <= 8 takes the small-M kernel (X resident in the LDS, in
 * chunks of K if it is larger than 150 KiB; TCSC lists streamed -- their padded 16-bit copy where there is one
 * and X fits the LDS whole), 8 < M <= 64 the small-tile kernel (one tile of
 * X, lists read from the TCSC arrays between the list cuts), everything else the large-M path (row sets).
 * Asynchronous: the kernels are enqueued on `stream` (a hipStream_t, NULL = null stream), no host
 * synchronisation, no allocation.
 * Device data are not validated.  Errors: EINVAL, ENOTUPLOADED, EHIP (launch failure).
 * Rounding: fp32 accumulation in an order fixed by (M, K, N), the matrix and the tuning
 * parameters; repeated calls give bit-identical results.  Integer-valued inputs small enough
 * for fp32 give exact results.
 * Two calls that use the same handle must be ordered (same stream, or an event between them):
 * they share the handle's workspace.
 */
int tstgemm(const float *X, const tcsc_t *t, const float *b, float *Y, int M, int K, int N, void *stream);

/*
 * Y = PReLU(X W + b): tstgemm() with the activation fused behind the bias add.  The paper fuses
 * PReLU into its vectorised kernels (Sec. 2 "Implementation Note", Sec. 4) without giving the
 * formula or the slope; here it is the usual one, PReLU(v) = v for v > 0 and alpha * v otherwise,
 * and the slopes are an input.
 * alpha: DEVICE fp32, alpha_count entries: 1 (one slope for all outputs) or N (alpha[n] for
 * column n of Y).  Everything else as for tstgemm().  The slope multiplication is the only
 * multiplication of the path; it rounds once in fp32.  Errors: as tstgemm(), and EINVAL for a
 * NULL alpha or an alpha_count other than 1 or N.
 */
int tstgemm_prelu(const float *X, const tcsc_t *t, const float *b, const float *alpha, int alpha_count, float *Y,
                  int M, int K, int N, void *stream);

/*
 * The matrix in the paper's "inverted index" encoding (Sec. 3): one list per column instead of two, +1 in row
 * i stored as i, -1 in row i as ~i (bitwise NOT), inside a column in ascending row order (the paper does not
 * state the order; this is the order of the lists that are merged).  col_start: HOST, N+1 entries;
 * index: HOST, nnz_pos + nnz_neg entries.  Computed on the host from the handle's arrays.
 */
int tcsc_signed_arrays(const tcsc_t *t, int32_t *col_start, int32_t *index);

/*
 * The matrix in the paper's "value compression" encoding (Sec. 3): five ternary entries per byte, the five
 * being the digits of a base-3 number.  What the paper leaves open is fixed like this: the five are
 * consecutive rows 5g .. 5g+4 of one column (rows >= K count as 0), an entry 0 / +1 / -1 is the digit 0 / 1 /
 * 2, the first row is the most significant digit (code = 81 d0 + 27 d1 + 9 d2 + 3 d3 + d4 <= 242), and the
 * codes are stored column after column.  codes: HOST, N * ceil(K/5) bytes, codes[n * ceil(K/5) + g].
 */
int tcsc_packed_codes(const tcsc_t *t, uint8_t *codes);

/*
 * Y = X W + b for M <= 8 from the inverted-index form in the device buffer (the decode kernel with one
 * signed list per column: the sign of an entry selects add or subtract, branch-free).  Arguments, rounding
 * and ordering rules as for tstgemm().  Errors: as tstgemm(), and EINVAL for M > 8.
 */
int tstgemm_signed(const float *X, const tcsc_t *t, const float *b, float *Y, int M, int K, int N, void *stream);

/*
 * Y = X W + b for M <= 8 from the value-compression form in the device buffer: every byte is decoded
 * through a 243-entry table (as in the paper) into five weights, and ALL entries take part in the sum,
 * the zeros as x * 0.  Unlike every other entry point this one therefore reads X entries whose weight is
 * zero: X must be finite.  Products with -1, 0, +1 are exact, so the rounding is that of the additions,
 * in an order fixed by (M, K, N) and the tuning parameters.  Arguments otherwise as for tstgemm() (it may
 * use the handle's workspace, so calls on one handle must be ordered).  Errors: as tstgemm(), and EINVAL
 * for M > 8.
 */
int tstgemm_packed(const float *X, const tcsc_t *t, const float *b, float *Y, int M, int K, int N, void *stream);

/*
 * Launch-shape overrides for the tiled paths (M > 8), for tuning runs and tests: columns per wavefront
 * (1, 2, 4 or 8; the small-tile kernel has 1, 2 and 4 and takes 8 as 4; 8 is the large-M path's wide
 * shape, which never slices K and needs a padded column count that is a multiple of 128, else it runs as 4),
 * number of K slices (1..8) computed by
 * different workgroups and summed in a fixed order (also the number of workgroups per column group of
 * tstgemm_packed()), and the largest number of row tiles of X packed and processed at a time (>= 1,
 * large-M path only).  0 restores the built-in choice for that parameter.  Process-wide.
 * Errors: EINVAL for a value outside the ranges above.
 */
int tstgemm_set_tuning(int cols_per_wave, int k_slices, int slab_tiles);

/*
 * Which copy of the lists the small-M kernel of tstgemm() reads when the matrix has both (K <= 65535): 0 (the
 * default) = the padded 16-bit copy, non-zero = the 32-bit TCSC arrays themselves.  For measurements and tests.  The
 * two deal the entries of a list to the lanes differently (8 or 4 consecutive ones per lane), so the fp32 rounding can
 * differ in the last bits; integer-valued inputs give the same, exact result.  Process-wide.  Always returns TSTGEMM_OK.
 */
int tstgemm_set_decode_lists(int wide);

/*
 * For benchmarks that must time one kernel: from now on every tstgemm() call records the
 * hipEvent_t `before` right before and `after` right after the launch of its main kernel
 * (the gather-add kernel; not the packing pre-pass and the split-K reduction of the tiled
 * paths), on the call's stream.  Both NULL switches this off (the default).  The events are
 * the caller's; a call with more than one slab of rows records them once per slab, so the pair
 * then brackets the last slab only.  Process-wide.  Errors: EINVAL if exactly one is NULL.
 */
int tstgemm_profile_events(void *before, void *after);

/*
 * Measurement probes (not part of the product path): what the machine delivers on the two resources the
 * kernels are priced against (operational intensity and peak, Sec. 4), for a benchmark that wants the
 * measured rate beside the datasheet one.  Both only enqueue one kernel on `stream`; the caller times it.
 *
 * tstgemm_probe_lds_read: 2 workgroups of 16 wavefronts per compute unit (the large-M kernel's occupancy), every
 * wavefront issues 8 * iters conflict-free 16-byte-per-lane LDS reads and nothing else.  *bytes_read (HOST,
 * may be NULL) receives the bytes all wavefronts read together.  1 <= iters <= 2^20, else EINVAL.
 *
 * tstgemm_probe_stream_read: reads buf (DEVICE, 16-byte aligned, bytes >= 16; whole 16-byte pieces are read,
 * a tail of bytes % 16 is not) once with 16-byte loads, grid-stride, 8 workgroups of 256 threads per
 * compute unit.  Errors: EINVAL, EHIP.
 */
int tstgemm_probe_lds_read(int iters, int64_t *bytes_read, void *stream);
int tstgemm_probe_stream_read(const void *buf, size_t bytes, void *stream);

/* Release the handle and its host arrays (not the device buffer).  NULL is allowed. */
void tcsc_destroy(tcsc_t *t);

/* Static text for a return code. */
const char *tcsc_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* TSTGEMM_H */
