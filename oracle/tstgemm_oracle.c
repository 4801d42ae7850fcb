/*
 * CPU oracle for the sparse ternary GEMM  Y = X W + b  -- TEST INFRASTRUCTURE ONLY.
 *
 * This file is the checker the GPU library is compared against.  It is plain, slow and
 * meant to be verified against the paper by eye.  Nothing of the product path may call
 * it: only the tests, the smoke check and the benchmark's cpu_baseline leg load it.
 * It shares no code, header, table or helper with the HIP sources.
 *
 * What it follows:
 *   - Eq. 1 (Sec. 2):  Y (MxN) = X (MxK) W (KxN, entries in {-1,0,+1}) + b (N), b added
 *     to every row of the product.
 *   - The TCSC format (Sec. 2): four integer arrays, col_start_pos / col_start_neg
 *     (N+1 column pointers each) and row_index_pos / row_index_neg (row numbers of the
 *     +1s / -1s, column after column).  The +1s of column j are
 *     row_index_pos[col_start_pos[j] .. col_start_pos[j+1]), likewise for the -1s.
 *   - The BaseTCSC algorithm (Sec. 2): for every output element, first add the X entries
 *     selected by the positive list, then subtract those selected by the negative list,
 *     then the bias.  Additions and subtractions only, no multiplication.
 *
 * Readings where the paper is silent: indices are 0-based int32, ascending inside a
 * column (Sec. 3, Blocking, relies on that order); X and Y are row-major;
 * the accumulator starts at zero and the bias is one final addition (the cost model
 * M N (1 + s K) of Sec. 2 counts exactly one add per output for it).
 *
 * Precision: accumulation in double.  Besides Yd (double) the routine returns
 *   A[m][n] = sum over the selected entries of |X[m][k]|  +  |b[n]|,
 * the magnitude the parity tolerance is scaled by.
 *
 * Optional activation (the paper fuses PReLU into its vectorised kernels, Sec. 2
 * "Implementation Note" and Sec. 4, without stating its formula or slope): oracle_prelu
 * applies the usual definition  PReLU(v) = v for v > 0, alpha * v otherwise  to a finished
 * Y, with one slope for all outputs or one per column of Y (output channel); the slopes are
 * inputs.  This is the only multiplication anywhere in the oracle.
 *
 * Parity pins (tests, CPU only): a hand-worked example, dense brute force through a
 * library matrix product on small and odd shapes, a sparse-library CSC construction for
 * the format, and the invariants W=0 => Y=b, Y(-W)-b = -(Y(W)-b), row permutation,
 * column independence, gather and row-sum special cases.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_BAD_VALUE -1 /* an entry of W outside {-1,0,+1} */
#define ORACLE_BAD_ARG -2

/* Number of +1 and -1 entries of a dense ternary W (row-major K x N). */
int oracle_tcsc_count(const int8_t *W, int K, int N, int64_t *nnz_pos, int64_t *nnz_neg)
{
    if (!W || K < 0 || N < 0 || !nnz_pos || !nnz_neg) return ORACLE_BAD_ARG;
    int64_t p = 0, q = 0;
    for (int64_t i = 0; i < (int64_t)K * N; ++i) {
        if (W[i] == 1) ++p;
        else if (W[i] == -1) ++q;
        else if (W[i] != 0) return ORACLE_BAD_VALUE;
    }
    *nnz_pos = p;
    *nnz_neg = q;
    return ORACLE_OK;
}

/*
 * TCSC construction (Sec. 2, the four arrays): scan column after column, inside a column
 * row after row; a +1 appends its row number to row_index_pos, a -1 to row_index_neg;
 * col_start_*[j] is the length of the respective list before column j, col_start_*[N]
 * its final length.
 */
int oracle_tcsc_build(const int8_t *W, int K, int N,
                      int32_t *col_start_pos, int32_t *col_start_neg,
                      int32_t *row_index_pos, int32_t *row_index_neg)
{
    if (!W || K < 0 || N < 0 || !col_start_pos || !col_start_neg) return ORACLE_BAD_ARG;
    int32_t p = 0, q = 0;
    for (int j = 0; j < N; ++j) {
        col_start_pos[j] = p;
        col_start_neg[j] = q;
        for (int k = 0; k < K; ++k) {
            int8_t w = W[(size_t)k * N + j];
            if (w == 1) row_index_pos[p++] = k;
            else if (w == -1) row_index_neg[q++] = k;
            else if (w != 0) return ORACLE_BAD_VALUE;
        }
    }
    col_start_pos[N] = p;
    col_start_neg[N] = q;
    return ORACLE_OK;
}

/* Inverse of the construction: write the dense ternary matrix the four arrays stand for. */
int oracle_tcsc_to_dense(const int32_t *col_start_pos, const int32_t *col_start_neg,
                         const int32_t *row_index_pos, const int32_t *row_index_neg,
                         int K, int N, int8_t *W)
{
    if (!W || K < 0 || N < 0) return ORACLE_BAD_ARG;
    for (int64_t i = 0; i < (int64_t)K * N; ++i) W[i] = 0;
    for (int j = 0; j < N; ++j) {
        for (int32_t t = col_start_pos[j]; t < col_start_pos[j + 1]; ++t)
            W[(size_t)row_index_pos[t] * N + j] = 1;
        for (int32_t t = col_start_neg[j]; t < col_start_neg[j + 1]; ++t)
            W[(size_t)row_index_neg[t] * N + j] = -1;
    }
    return ORACLE_OK;
}

/* One output element in BaseTCSC order: positives added, negatives subtracted, bias last. */
static void oracle_element(const float *x_row,
                           const int32_t *col_start_pos, const int32_t *col_start_neg,
                           const int32_t *row_index_pos, const int32_t *row_index_neg,
                           const float *b, int n, double *y, double *a)
{
    double acc = 0.0, mag = 0.0;
    for (int32_t t = col_start_pos[n]; t < col_start_pos[n + 1]; ++t) {
        double v = (double)x_row[row_index_pos[t]];
        acc += v;
        mag += fabs(v);
    }
    for (int32_t t = col_start_neg[n]; t < col_start_neg[n + 1]; ++t) {
        double v = (double)x_row[row_index_neg[t]];
        acc -= v;
        mag += fabs(v);
    }
    double bias = b ? (double)b[n] : 0.0;
    *y = acc + bias;
    if (a) *a = mag + fabs(bias);
}

/*
 * Rows rows[0..n_rows) of Y (rows == NULL: rows 0..n_rows-1, i.e. n_rows = M gives all of
 * Y).  Yd and A are n_rows x N, row-major; A may be NULL.  X is M x K row-major, b has N
 * entries or is NULL (taken as zero).  threads <= 0 leaves the OpenMP default.
 * Returns the number of threads used, or a negative error code.
 */
int oracle_tstgemm_rows(const float *X,
                        const int32_t *col_start_pos, const int32_t *col_start_neg,
                        const int32_t *row_index_pos, const int32_t *row_index_neg,
                        const float *b, const int32_t *rows, int n_rows,
                        int M, int K, int N, double *Yd, double *A, int threads)
{
    if (!X || !Yd || !col_start_pos || !col_start_neg || M < 0 || K < 0 || N < 0 || n_rows < 0)
        return ORACLE_BAD_ARG;
    if (!rows && n_rows > M) return ORACLE_BAD_ARG;
    int used = 1;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
    used = omp_get_max_threads();
#endif
    int64_t total = (int64_t)n_rows * N;
    /* Few rows (decode shapes): spread the columns over the threads instead of the rows. */
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < total; ++e) {
        int r = (int)(e / N), n = (int)(e % N);
        int m = rows ? rows[r] : r;
        oracle_element(X + (size_t)m * K, col_start_pos, col_start_neg, row_index_pos, row_index_neg,
                       b, n, &Yd[e], A ? &A[e] : 0);
    }
    return used;
}

/* Sampled outputs: Yd[i], A[i] for the element (ms[i], ns[i]), i < n_points. */
int oracle_tstgemm_points(const float *X,
                          const int32_t *col_start_pos, const int32_t *col_start_neg,
                          const int32_t *row_index_pos, const int32_t *row_index_neg,
                          const float *b, const int32_t *ms, const int32_t *ns, int64_t n_points,
                          int M, int K, int N, double *Yd, double *A)
{
    if (!X || !Yd || !ms || !ns || M < 0 || K < 0 || N < 0) return ORACLE_BAD_ARG;
    for (int64_t i = 0; i < n_points; ++i)
        if (ms[i] < 0 || ms[i] >= M || ns[i] < 0 || ns[i] >= N) return ORACLE_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_points; ++i)
        oracle_element(X + (size_t)ms[i] * K, col_start_pos, col_start_neg, row_index_pos, row_index_neg,
                       b, ns[i], &Yd[i], A ? &A[i] : 0);
    return ORACLE_OK;
}

/*
 * PReLU on a finished block of Y (n_rows x N, row-major, in place): v > 0 stays, otherwise
 * v becomes alpha * v.  alpha_count == 1: alpha[0] for every output; alpha_count == N: alpha[n]
 * for column n.  A (may be NULL) is scaled by max(1, |alpha|): the function is Lipschitz with
 * that constant, so an error bound on v carries over with this factor.
 */
int oracle_prelu(double *Yd, double *A, int n_rows, int N, const float *alpha, int alpha_count)
{
    if (!Yd || !alpha || n_rows < 0 || N < 0 || (alpha_count != 1 && alpha_count != N)) return ORACLE_BAD_ARG;
    for (int r = 0; r < n_rows; ++r) {
        for (int n = 0; n < N; ++n) {
            double a = (double)alpha[alpha_count == 1 ? 0 : n];
            double v = Yd[(size_t)r * N + n];
            if (!(v > 0.0)) Yd[(size_t)r * N + n] = a * v;
            if (A && fabs(a) > 1.0) A[(size_t)r * N + n] *= fabs(a);
        }
    }
    return ORACLE_OK;
}
