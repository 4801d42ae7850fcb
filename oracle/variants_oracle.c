/*
 * CPU oracle for the two alternative encodings of the ternary matrix W that the paper tried
 * next to TCSC (Sec. 3, "Inverted Index" and "Value Compression") -- TEST INFRASTRUCTURE ONLY.
 * Same rules as tstgemm_oracle.c: plain, slow, fp64, shares nothing with the HIP sources, and
 * only the tests, the smoke check and the benchmark's cpu_baseline leg may load it.
 *
 * Both encodings stand for the same W, so the product has the plain definition of Eq. 1,
 * Y = X W + b; the routines below nevertheless walk the encoded data themselves, in the
 * order the encoding gives, so that the encoding (not just the result) is what gets checked.
 *
 * 1. Inverted index: the two sign lists of a column are merged into one; an entry +1 in row i
 *    is stored as i, an entry -1 in row i as ~i (bitwise NOT, a negative number).  One pointer
 *    array of N+1 entries instead of two.  Reading where the paper is silent: inside a column
 *    the merged list is ascending in the row number (the order of the TCSC lists it merges).
 *
 * 2. Value compression: five ternary entries in one byte, the five taken as the digits of a
 *    base-3 number (3^5 = 243 <= 256).  Readings where the paper is silent: the five are
 *    consecutive ROWS of one column (TCSC is column-wise); rows beyond K count as 0; the digit
 *    of an entry is 0 for 0, 1 for +1, 2 for -1 (so an all-zero group has code 0); the first
 *    (lowest) row is the most significant digit, as one writes a number; codes are stored column
 *    after column, ceil(K/5) bytes per column.  Decoding goes through a table of the 243
 *    five-tuples, as in the paper.
 *
 * Parity pins (tests, CPU only): a hand-worked example for both encodings, hand-computed codes
 * of single groups, round trips through the dense matrix, the count of distinct codes, and
 * agreement of the products with the TCSC oracle (bit for bit on integer inputs).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

#define ORACLE_OK 0
#define ORACLE_BAD_VALUE -1
#define ORACLE_BAD_ARG -2

/* ---------------------------------------------------------------- inverted index */

/* TCSC -> merged signed lists.  col_start: N+1 entries; index: nnz_pos + nnz_neg entries. */
int oracle_signed_build(const int32_t *col_start_pos, const int32_t *col_start_neg,
                        const int32_t *row_index_pos, const int32_t *row_index_neg,
                        int N, int32_t *col_start, int32_t *index)
{
    if (!col_start_pos || !col_start_neg || !col_start || N < 0) return ORACLE_BAD_ARG;
    int32_t out = 0;
    for (int j = 0; j < N; ++j) {
        col_start[j] = out;
        int32_t p = col_start_pos[j], p1 = col_start_pos[j + 1];
        int32_t q = col_start_neg[j], q1 = col_start_neg[j + 1];
        while (p < p1 || q < q1) {
            /* the smaller row goes first; a row is never in both lists */
            if (q >= q1 || (p < p1 && row_index_pos[p] < row_index_neg[q])) index[out++] = row_index_pos[p++];
            else index[out++] = ~row_index_neg[q++];
        }
    }
    col_start[N] = out;
    return ORACLE_OK;
}

/* Dense W (row-major K x N) of a merged signed list. */
int oracle_signed_to_dense(const int32_t *col_start, const int32_t *index, int K, int N, int8_t *W)
{
    if (!col_start || !W || K < 0 || N < 0) return ORACLE_BAD_ARG;
    for (int64_t i = 0; i < (int64_t)K * N; ++i) W[i] = 0;
    for (int j = 0; j < N; ++j)
        for (int32_t t = col_start[j]; t < col_start[j + 1]; ++t) {
            int32_t e = index[t];
            int32_t row = e < 0 ? ~e : e;
            if (row >= K) return ORACLE_BAD_VALUE;
            W[(size_t)row * N + j] = e < 0 ? -1 : 1;
        }
    return ORACLE_OK;
}

/* Y = X W + b from the merged lists: one loop per output, the sign decoded per entry; bias last.
 * Yd, A: M x N (A as in the TCSC oracle: sum of |X| over the selected entries + |b|; may be NULL). */
int oracle_tstgemm_signed(const float *X, const int32_t *col_start, const int32_t *index, const float *b,
                          int M, int K, int N, double *Yd, double *A)
{
    if (!X || !col_start || !Yd || M < 0 || K < 0 || N < 0) return ORACLE_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < (int64_t)M * N; ++e) {
        int m = (int)(e / N), n = (int)(e % N);
        double acc = 0.0, mag = 0.0;
        for (int32_t t = col_start[n]; t < col_start[n + 1]; ++t) {
            int32_t s = index[t];
            double v = (double)X[(size_t)m * K + (s < 0 ? ~s : s)];
            if (s < 0) acc -= v; else acc += v;
            mag += fabs(v);
        }
        double bias = b ? (double)b[n] : 0.0;
        Yd[e] = acc + bias;
        if (A) A[e] = mag + fabs(bias);
    }
    return ORACLE_OK;
}

/* ---------------------------------------------------------------- value compression */

static int digit_of(int8_t w) { return w == 0 ? 0 : w == 1 ? 1 : w == -1 ? 2 : -1; }

/* Dense W (row-major K x N) -> codes[n * G + g], G = ceil(K / 5); group g of column n holds rows 5g .. 5g+4. */
int oracle_pack5(const int8_t *W, int K, int N, uint8_t *codes)
{
    if (!W || !codes || K < 0 || N < 0) return ORACLE_BAD_ARG;
    int G = (K + 4) / 5;
    for (int n = 0; n < N; ++n)
        for (int g = 0; g < G; ++g) {
            int code = 0;
            for (int j = 0; j < 5; ++j) {
                int k = 5 * g + j;
                int d = k < K ? digit_of(W[(size_t)k * N + n]) : 0;
                if (d < 0) return ORACLE_BAD_VALUE;
                code = code * 3 + d;   /* first row = most significant digit */
            }
            codes[(size_t)n * G + g] = (uint8_t)code;
        }
    return ORACLE_OK;
}

/* The decoding table: tuple[c][j] is the entry (as -1, 0, +1) of row j of a group with code c, c < 243. */
static void five_tuples(int8_t tuple[243][5])
{
    for (int c = 0; c < 243; ++c) {
        int rest = c;
        for (int j = 4; j >= 0; --j) {
            int d = rest % 3;
            rest /= 3;
            tuple[c][j] = d == 0 ? 0 : d == 1 ? 1 : -1;
        }
    }
}

int oracle_unpack5(const uint8_t *codes, int K, int N, int8_t *W)
{
    if (!W || !codes || K < 0 || N < 0) return ORACLE_BAD_ARG;
    int8_t tuple[243][5];
    five_tuples(tuple);
    int G = (K + 4) / 5;
    for (int n = 0; n < N; ++n)
        for (int g = 0; g < G; ++g) {
            uint8_t c = codes[(size_t)n * G + g];
            if (c >= 243) return ORACLE_BAD_VALUE;
            for (int j = 0; j < 5; ++j) {
                int k = 5 * g + j;
                if (k < K) W[(size_t)k * N + n] = tuple[c][j];
                else if (tuple[c][j] != 0) return ORACLE_BAD_VALUE;   /* padding rows must be zero */
            }
        }
    return ORACLE_OK;
}

/* Y = X W + b from the codes: every group is decoded through the table, its non-zero entries are added or
 * subtracted in row order (zero entries are skipped: their X values are not read); bias last. */
int oracle_tstgemm_packed(const float *X, const uint8_t *codes, const float *b, int M, int K, int N, double *Yd,
                          double *A)
{
    if (!X || !codes || !Yd || M < 0 || K < 0 || N < 0) return ORACLE_BAD_ARG;
    int8_t tuple[243][5];
    five_tuples(tuple);
    int G = (K + 4) / 5;
    for (int64_t i = 0; i < (int64_t)N * G; ++i)
        if (codes[i] >= 243) return ORACLE_BAD_VALUE;
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < (int64_t)M * N; ++e) {
        int m = (int)(e / N), n = (int)(e % N);
        double acc = 0.0, mag = 0.0;
        for (int g = 0; g < G; ++g) {
            const int8_t *w = tuple[codes[(size_t)n * G + g]];
            for (int j = 0; j < 5; ++j) {
                if (w[j] == 0) continue;
                double v = (double)X[(size_t)m * K + 5 * g + j];
                if (w[j] > 0) acc += v; else acc -= v;
                mag += fabs(v);
            }
        }
        double bias = b ? (double)b[n] : 0.0;
        Yd[e] = acc + bias;
        if (A) A[e] = mag + fabs(bias);
    }
    return ORACLE_OK;
}
