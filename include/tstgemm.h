/*
 * tstgemm -- sparse ternary GEMM  Y = X W + b  for one AMD MI355X (gfx950).
 *
 * C ABI of libtstgemm.so.  Plain pointers and sizes only; every pointer argument says
 * whether it is HOST or DEVICE memory.  All functions return 0 (TSTGEMM_OK) or a negative
 * TSTGEMM_E* code; tcsc_strerror() turns a code into text.  No function throws, aborts or
 * prints.  The library keeps no mutable global state: everything a call depends on is in its
 * arguments and in the handle (what the library caches per device -- the number of compute units, a
 * kernel attribute that has been set -- is read-only information about the machine).
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
#define TSTGEMM_ETOOBIG (-6)      /* more than 2^31-1 non-zero entries (both signs together), or K >= 2^31 */
#define TSTGEMM_ENOFORM (-7)      /* the device form this call reads was not selected for the upload
                                     (tcsc_select_forms) */
#define TSTGEMM_EWORKSPACE (-8)   /* the call needs scratch memory and has none (no workspace argument and none in
                                     the handle), or less than tstgemm_workspace_bytes() gives as the minimum */
#define TSTGEMM_ESCRATCH (-9)     /* tstgemm_noalloc(): the call needs more scratch memory than the library's static
                                     buffer (TSTGEMM_NOALLOC_SCRATCH_BYTES) holds */

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
 *                                             Inside a column's list the entries are NOT ascending: their order (a sum
 *                                             does not care) is chosen so that the sixteen lanes that gather together get
 *                                             rows that differ modulo 16, i.e. lie in different LDS banks; the pad entries
 *                                             can be anywhere in the list.
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
 *   workspace  bytes  [workspace_bytes]       scratch for calls that bring none of their own: split-K partial sums and
 *                                             a tiled, transposed copy of (a slab of rows of) X; 160 MiB, or 32 MiB + one
 *                                             tile of 256 rows over the padded K if that is larger
 * n_pad = N rounded up to a multiple of 64; columns >= N have empty sets.
 * Which of these the buffer holds is the handle's choice of forms (tcsc_select_forms; default: all); a form
 * that is not selected has offset 0 and takes no room.  The four TCSC arrays are always there.
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
    uint32_t forms;                 /* TCSC_FORM_* bits of what the buffer holds */
} tcsc_layout_t;

/*
 * Device forms besides the four TCSC arrays (which are always uploaded: the decode kernel of tstgemm() for
 * M <= 8 reads them, and every other form is derived from them on the GPU):
 */
#define TCSC_FORM_ROWSETS 1u     /* masks: the large-M path of tstgemm(), M > 64 */
#define TCSC_FORM_CUTS 2u        /* list_cuts: the small-tile path of tstgemm(), 8 < M <= 64 (a matrix with 2^30 or more
                                    entries of one sign takes the large-M path for these M too: ROWSETS) */
#define TCSC_FORM_LISTS16 4u     /* padded 16-bit lists (only where K <= 65535): M <= 8 reads half the bytes */
#define TCSC_FORM_SIGNED 8u      /* signed_index: tstgemm_signed() */
#define TCSC_FORM_PACKED 16u     /* packed: tstgemm_packed(); built from the row sets, so it selects ROWSETS too */
#define TCSC_FORM_WORKSPACE 32u  /* scratch inside the buffer, for calls without a workspace argument */
#define TCSC_FORM_ALL 63u

/*
 * Choose what tcsc_upload() puts into the device buffer (a new handle has TCSC_FORM_ALL).  Changes
 * tcsc_device_bytes() and tcsc_layout(); a handle that was already uploaded must be uploaded again.  A matrix that
 * serves one shape of X needs one form: e.g. ROWSETS alone for M > 64 with a caller-supplied workspace
 * (tstgemm_ex) is 16 bytes per column and 64 rows of W beside the TCSC arrays.
 * Errors: EINVAL for a NULL handle or bits outside TCSC_FORM_ALL.
 */
int tcsc_select_forms(tcsc_t *t, uint32_t forms);

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
 * X, lists read from the TCSC arrays between the list cuts; not for matrices with 2^30 or more entries of one sign,
 * whose lists its 32-bit byte offsets do not reach), everything else the large-M path (row sets).
 * Asynchronous: the kernels are enqueued on `stream` (a hipStream_t, NULL = null stream), no host
 * synchronisation, no allocation.
 * Device data are not validated.  Errors: EINVAL, ENOTUPLOADED, ENOFORM, EWORKSPACE, EHIP (launch failure).
 * Rounding: fp32 accumulation in an order fixed by (M, K, N), the matrix, the launch-shape options and the
 * size of the workspace; repeated calls give bit-identical results.  Integer-valued inputs small enough
 * for fp32 give exact results.
 * Scratch memory (M > 8): this call uses the workspace inside the handle's device buffer (TCSC_FORM_WORKSPACE),
 * so two calls on the same handle must be ordered (same stream, or an event between them).  tstgemm_ex() takes
 * a workspace argument instead.
 */
int tstgemm(const float *X, const tcsc_t *t, const float *b, float *Y, int M, int K, int N, void *stream);

/*
 * Scratch memory a call with these dimensions needs (the tiled, transposed copy of X of the paths for M > 8 and
 * the partial sums of K slices; Sec. 3 "Blocking" is where the tiles come from).  *min_bytes: the least a call
 * runs with (one row tile of X over the padded K; rows then go through in slabs and K is not sliced);
 * *best_bytes: what it takes to run every shape the library would choose by itself in one slab.  M <= 8: 0
 * and the (small) partial sums tstgemm_packed() may use.  Either pointer may be NULL.  Errors: EINVAL.
 */
int tstgemm_workspace_bytes(int M, int K, int N, size_t *min_bytes, size_t *best_bytes);

/*
 * Everything a call can be told beyond its operands.  Zero-initialise, set struct_size = sizeof(tstgemm_opts_t)
 * and the fields that matter; a zeroed struct (with struct_size) makes tstgemm_ex() the same as tstgemm().
 */
typedef struct tstgemm_opts {
    size_t struct_size;
    int encoding;            /* 0: TCSC (as tstgemm), 1: inverted index (as tstgemm_signed, M <= 8),
                                2: value compression (as tstgemm_packed, M <= 8, X finite) */
    int alpha_count;         /* 1 or N when alpha is given */
    const float *alpha;      /* DEVICE PReLU slopes (as tstgemm_prelu; encoding 0 only) or NULL for none */
    void *workspace;         /* DEVICE scratch, 256-byte aligned, owned by the caller, or NULL for the handle's own.
                                Used from the moment the call is enqueued until its last kernel has finished; calls
                                whose kernels may overlap (different streams) need different workspaces, calls on one
                                stream can share one across any number of matrices */
    size_t workspace_bytes;  /* at least the min_bytes of tstgemm_workspace_bytes(), else EWORKSPACE */
    /* Launch-shape overrides for the tiled paths (M > 8), for tuning runs and tests; 0 = the built-in choice.
     * cols_per_wave: 1, 2, 4 or 8 columns of Y per wavefront (the small-tile kernel has 1, 2, 4 and takes 8 as 4; 8 is
     * the large-M path's wide shape, which needs a padded column count that is a multiple of 128, else it runs as 4);
     * k_slices: 1..8 slices of K computed by different workgroups and summed in slice order (also the workgroups per
     * column group of encoding 2); slab_tiles: at most this many row tiles of X packed and processed at a time. */
    int cols_per_wave, k_slices, slab_tiles;
    int list_walk;           /* 8 < M <= 64, for tuning runs and tests: 0 = the built-in choice by the density of W,
                                1 = the plain walk of the lists (best on short lists), 2 = the walk that requests the
                                entries of a list two steps ahead (best from about 40 entries per list and 256 rows of
                                W on).  Same sums, added in a different order */
    int decode_wide_lists;   /* != 0: M <= 8 reads the 32-bit TCSC lists even where the padded 16-bit copy exists.  The two
                                deal the entries of a list to the lanes differently, so fp32 rounding can differ in the
                                last bits; integer-valued inputs give the same, exact result */
    void *event_before, *event_after;   /* hipEvent_t pair (both or neither), recorded on the call's stream right before
                                and after the launch of the main (gather-add) kernel, not around the packing
                                pre-pass and the reduction of K slices; a call with several slabs of rows records
                                them once per slab, so the pair then brackets the last slab.  The caller's. */
} tstgemm_opts_t;

/*
 * Y = X W + b (Eq. 1) with options: tstgemm(), tstgemm_prelu(), tstgemm_signed() and tstgemm_packed() are this call
 * with the options they stand for.  opts may be NULL (= tstgemm()).  Operands, rounding and asynchrony as for
 * tstgemm().  Errors: as tstgemm(); EINVAL also for a struct_size that is not this header's, an unknown encoding,
 * an option outside its range, exactly one event, alpha with encoding != 0, or a misaligned workspace.
 */
int tstgemm_ex(const float *X, const tcsc_t *t, const float *b, float *Y, int M, int K, int N,
               const tstgemm_opts_t *opts, void *stream);

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
 * tstgemm() for callers that cannot allocate device memory and have no workspace to pass: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same operands, result and errors as tstgemm_ex()
 * with default options and a workspace of TSTGEMM_NOALLOC_SCRATCH_BYTES, but the workspace is a static device array
 * inside the library (one per GPU, held until the process ends), so the handle needs no TCSC_FORM_WORKSPACE and the
 * call makes no allocation of any kind.  Limit: the minimum of tstgemm_workspace_bytes(M, K, N) must fit the array
 * (a row tile of 256 rows over K up to 65536; any M -- taller X goes through in slabs, and K is sliced as far
 * as the rest of the array holds partial sums), else ESCRATCH and nothing is launched.  All calls on one GPU share
 * that GPU's array: calls that may overlap (different streams without an event between them, different threads)
 * race on it -- order them, or use tstgemm_ex() with separate workspaces.  The array keeps the last call's contents;
 * no call depends on them.  The first call on a device looks the array's address up (once per device); make that
 * call outside a graph capture.
 */
#define TSTGEMM_NOALLOC_SCRATCH_BYTES ((size_t)64 << 20)
int tstgemm_noalloc(const float *X, const tcsc_t *t, const float *b, float *Y, int M, int K, int N, void *stream);

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
 * in an order fixed by (M, K, N) and the options.  Arguments otherwise as for tstgemm() (it may
 * use the handle's workspace, so calls on one handle must be ordered).  Errors: as tstgemm(), and EINVAL
 * for M > 8.
 */
int tstgemm_packed(const float *X, const tcsc_t *t, const float *b, float *Y, int M, int K, int N, void *stream);

/*
 * Measurement probes (not part of the product path): what the machine delivers on the resources the
 * kernels are priced against (operational intensity and peak, Sec. 4), for a benchmark that wants the
 * measured rate beside the datasheet one.  Each only enqueues one kernel on `stream`; the caller times it.
 *
 * tstgemm_probe_lds_read: 2 workgroups of 16 wavefronts per compute unit (the large-M kernel's occupancy), every
 * wavefront issues 8 * iters conflict-free 16-byte-per-lane LDS reads and nothing else.  *bytes_read (HOST,
 * may be NULL) receives the bytes all wavefronts read together.  1 <= iters <= 2^20, else EINVAL.
 *
 * tstgemm_probe_stream_read: reads buf (DEVICE, 16-byte aligned, bytes >= 16; whole 16-byte pieces are read,
 * a tail of bytes % 16 is not) once with 16-byte loads, grid-stride, 8 workgroups of 256 threads per
 * compute unit.  Errors: EINVAL, EHIP.
 *
 * tstgemm_probe_tile_copy: the tile exchange of the tiled paths (the blocks of Sec. 3 "Blocking" on their way into
 * the LDS) and nothing else: 2 workgroups of 16 wavefronts per compute unit, each copies `iters` times a 64 KiB
 * piece of buf (DEVICE, 16-byte aligned, bytes >= 65536; the whole 64 KiB pieces of it, taken in turn, workgroup w
 * starting at piece w) into its LDS -- 16-byte loads, barrier, 16-byte LDS writes, barrier.  With a buffer of a few
 * MiB the pieces come from the L2s, as the packed copy of X does in a call.  *bytes_copied (HOST, may be NULL)
 * receives the bytes all workgroups copy together.  1 <= iters <= 2^20.  Errors: EINVAL, EHIP.
 */
int tstgemm_probe_lds_read(int iters, int64_t *bytes_read, void *stream);
int tstgemm_probe_stream_read(const void *buf, size_t bytes, void *stream);
int tstgemm_probe_tile_copy(const void *buf, size_t bytes, int iters, int64_t *bytes_copied, void *stream);

/* Release the handle and its host arrays (not the device buffer).  NULL is allowed. */
void tcsc_destroy(tcsc_t *t);

/* Static text for a return code. */
const char *tcsc_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* TSTGEMM_H */
