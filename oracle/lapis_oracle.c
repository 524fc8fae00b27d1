/*
 * CPU oracle for the CSR sparse matrix-vector product and its multi-vector
 * form.  TEST INFRASTRUCTURE ONLY: tests, the smoke check and the bench's
 * cpu_baseline leg may call it; the product path never does, and nothing here
 * shares code, headers, tables or helpers with the GPU library.
 *
 * What it computes is the plain definition the paper gives in Section 6.2
 * (y := A x, A in CSR, x and y dense), walked with the row / entry loop nest
 * of Section 4.2 ("Parallelism estimation": for each row i, begin =
 * offsets[i], end = offsets[i+1], entries begin..end-1), serial, entries taken
 * left to right.  The scaling y = alpha*A*x + beta*y0 is the BLAS-style
 * extension of the problem statement; beta == 0 means y0 is never read.
 *
 * Precision: every sum and product is formed in double.  For float matrices
 * the inputs are promoted exactly and the result is rounded to float once.
 * Build with -ffp-contract=off so that no fused multiply-add is introduced.
 *
 * Beside each result the oracle returns (|A||x|)_i = sum_j |a_ij| |x_j|, the
 * quantity the floating-point tolerance is stated in.
 *
 * The row-partition reference at the end is the integer definition of the
 * analysis pass (stream chunks, row bins by length, stable row lists,
 * equal-nnz tiles over the long rows), written as plain loops.  Its constants are arguments, so
 * this file carries no copy of the library's header.
 *
 * Pins (tests marked "not gpu"): dense brute force on tiny matrices,
 * identity and diagonal matrices, the 5-point Laplacian's closed forms on
 * constant and linear grid functions, exact integer-valued cases, linearity,
 * SpMM column == SpMV, library cross-checks (SciPy / PyTorch CPU), the
 * transposed product against dense A^T, the adjoint identity and symmetric
 * matrices, and
 * structural invariants of the partition.  No function here is unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

/* ---- SpMV, double matrix ------------------------------------------------ */
void oracle_spmv_f64(int64_t nrows, const int32_t *rowptr, const int32_t *colidx,
                     const double *vals, const double *x, double alpha, double beta,
                     const double *y0, double *y, double *absAx)
{
    for (int64_t i = 0; i < nrows; ++i) {
        double s = 0.0, t = 0.0;
        for (int64_t j = rowptr[i]; j < rowptr[i + 1]; ++j) {
            double a = vals[j], b = x[colidx[j]];
            s += a * b;
            t += fabs(a) * fabs(b);
        }
        y[i] = (beta == 0.0) ? alpha * s : alpha * s + beta * y0[i];
        if (absAx) absAx[i] = t;
    }
}

/* ---- SpMV, float matrix: double arithmetic, one final rounding ---------- */
void oracle_spmv_f32(int64_t nrows, const int32_t *rowptr, const int32_t *colidx,
                     const float *vals, const float *x, double alpha, double beta,
                     const float *y0, float *y, double *absAx)
{
    for (int64_t i = 0; i < nrows; ++i) {
        double s = 0.0, t = 0.0;
        for (int64_t j = rowptr[i]; j < rowptr[i + 1]; ++j) {
            double a = (double)vals[j], b = (double)x[colidx[j]];
            s += a * b;
            t += fabs(a) * fabs(b);
        }
        double r = (beta == 0.0) ? alpha * s : alpha * s + beta * (double)y0[i];
        y[i] = (float)r;
        if (absAx) absAx[i] = t;
    }
}

/* ---- transposed product: y = alpha * A^T x + beta * y0 --------------------
 * The column-wise (CSC) traversal of the loop pattern of Section 4.2: the CSR arrays of A are
 * the CSC arrays of A^T, so entry j of row i contributes vals[j] * x[i] to y[colidx[j]].
 * Definition written out: the sums are accumulated in double in row order, then scaled once.
 * x has nrows elements, y0 / y / absATx have ncols; acc is caller scratch of 2*ncols doubles. */
void oracle_spmv_transpose_f64(int64_t nrows, int64_t ncols, const int32_t *rowptr, const int32_t *colidx,
                               const double *vals, const double *x, double alpha, double beta,
                               const double *y0, double *y, double *absATx, double *acc)
{
    double *s = acc, *t = acc + ncols;
    for (int64_t c = 0; c < ncols; ++c) s[c] = t[c] = 0.0;
    for (int64_t i = 0; i < nrows; ++i)
        for (int64_t j = rowptr[i]; j < rowptr[i + 1]; ++j) {
            s[colidx[j]] += vals[j] * x[i];
            t[colidx[j]] += fabs(vals[j]) * fabs(x[i]);
        }
    for (int64_t c = 0; c < ncols; ++c) {
        y[c] = (beta == 0.0) ? alpha * s[c] : alpha * s[c] + beta * y0[c];
        if (absATx) absATx[c] = t[c];
    }
}

void oracle_spmv_transpose_f32(int64_t nrows, int64_t ncols, const int32_t *rowptr, const int32_t *colidx,
                               const float *vals, const float *x, double alpha, double beta,
                               const float *y0, float *y, double *absATx, double *acc)
{
    double *s = acc, *t = acc + ncols;
    for (int64_t c = 0; c < ncols; ++c) s[c] = t[c] = 0.0;
    for (int64_t i = 0; i < nrows; ++i)
        for (int64_t j = rowptr[i]; j < rowptr[i + 1]; ++j) {
            s[colidx[j]] += (double)vals[j] * (double)x[i];
            t[colidx[j]] += fabs((double)vals[j]) * fabs((double)x[i]);
        }
    for (int64_t c = 0; c < ncols; ++c) {
        double r = (beta == 0.0) ? alpha * s[c] : alpha * s[c] + beta * (double)y0[c];
        y[c] = (float)r;
        if (absATx) absATx[c] = t[c];
    }
}

/* ---- explicit transposition: CSR arrays of A^T ---------------------------
 * The textbook counting transposition: count the entries of every column, prefix-sum the
 * counts into tptr, then walk A in row order and append each entry to its column.  Walking in
 * row order makes the result unique: inside row c of A^T the entries are ordered by (row of A,
 * position inside that row), duplicates included.  tptr has ncols+1 elements, tidx and tvals
 * have nnz; esize is the size of one value in bytes (values are moved, not computed with). */
void oracle_transpose(int64_t nrows, int64_t ncols, const int32_t *rowptr, const int32_t *colidx,
                      const void *vals, int64_t esize, int32_t *tptr, int32_t *tidx, void *tvals)
{
    for (int64_t c = 0; c <= ncols; ++c) tptr[c] = 0;
    for (int64_t j = 0; j < rowptr[nrows]; ++j) tptr[colidx[j] + 1] += 1;
    for (int64_t c = 0; c < ncols; ++c) tptr[c + 1] += tptr[c];
    /* tptr[c] is advanced while filling and restored by the shift afterwards */
    for (int64_t i = 0; i < nrows; ++i)
        for (int64_t j = rowptr[i]; j < rowptr[i + 1]; ++j) {
            const int64_t p = tptr[colidx[j]]++;
            tidx[p] = (int32_t)i;
            for (int64_t b = 0; b < esize; ++b)
                ((unsigned char *)tvals)[p * esize + b] = ((const unsigned char *)vals)[j * esize + b];
        }
    for (int64_t c = ncols; c > 0; --c) tptr[c] = tptr[c - 1];
    tptr[0] = 0;
}

/* ---- Batched GEMM (Section 5, the batched kernel the paper lowers with the batch dimension
 * vectorised): for every b < batch, C[b] = alpha * A[b] * B[b] + beta * C0[b] with A[b] m x k,
 * B[b] k x n, C[b] m x n, each matrix row-major and the matrices of an operand back to back.
 * The plain definition: one dot product per element, summed left to right in double (f32
 * operands promoted, the result rounded once).  absAB (may be NULL) receives sum |a||b| for the
 * tolerance.  beta == 0: C0 is not read. ---------------------------------------------------- */
void oracle_batched_gemm_f64(int64_t batch, int64_t m, int64_t n, int64_t k, double alpha, const double *A,
                             const double *B, double beta, const double *C0, double *C, double *absAB)
{
    for (int64_t b = 0; b < batch; ++b)
        for (int64_t i = 0; i < m; ++i)
            for (int64_t j = 0; j < n; ++j) {
                double s = 0.0, t = 0.0;
                for (int64_t l = 0; l < k; ++l) {
                    double x = A[(b * m + i) * k + l], y = B[(b * k + l) * n + j];
                    s += x * y;
                    t += fabs(x) * fabs(y);
                }
                int64_t at = (b * m + i) * n + j;
                C[at] = (beta == 0.0) ? alpha * s : alpha * s + beta * C0[at];
                if (absAB) absAB[at] = t;
            }
}

void oracle_batched_gemm_f32(int64_t batch, int64_t m, int64_t n, int64_t k, double alpha, const float *A,
                             const float *B, double beta, const float *C0, float *C, double *absAB)
{
    for (int64_t b = 0; b < batch; ++b)
        for (int64_t i = 0; i < m; ++i)
            for (int64_t j = 0; j < n; ++j) {
                double s = 0.0, t = 0.0;
                for (int64_t l = 0; l < k; ++l) {
                    double x = (double)A[(b * m + i) * k + l], y = (double)B[(b * k + l) * n + j];
                    s += x * y;
                    t += fabs(x) * fabs(y);
                }
                int64_t at = (b * m + i) * n + j;
                double r = (beta == 0.0) ? alpha * s : alpha * s + beta * (double)C0[at];
                C[at] = (float)r;
                if (absAB) absAB[at] = t;
            }
}

/* ---- SpMM: Y = alpha*A*X + beta*Y0, X, Y0, Y row-major with leading
 * dimensions ldx, ldy (Y0 and Y share ldy); absAX is nrows*k contiguous.
 * Column c is by definition the SpMV with column c of X. ------------------- */
void oracle_spmm_f64(int64_t nrows, int64_t k, const int32_t *rowptr, const int32_t *colidx,
                     const double *vals, const double *X, int64_t ldx, double alpha, double beta,
                     const double *Y0, double *Y, int64_t ldy, double *absAX)
{
    for (int64_t i = 0; i < nrows; ++i) {
        for (int64_t c = 0; c < k; ++c) {
            double s = 0.0, t = 0.0;
            for (int64_t j = rowptr[i]; j < rowptr[i + 1]; ++j) {
                double a = vals[j], b = X[(int64_t)colidx[j] * ldx + c];
                s += a * b;
                t += fabs(a) * fabs(b);
            }
            Y[i * ldy + c] = (beta == 0.0) ? alpha * s : alpha * s + beta * Y0[i * ldy + c];
            if (absAX) absAX[i * k + c] = t;
        }
    }
}

void oracle_spmm_f32(int64_t nrows, int64_t k, const int32_t *rowptr, const int32_t *colidx,
                     const float *vals, const float *X, int64_t ldx, double alpha, double beta,
                     const float *Y0, float *Y, int64_t ldy, double *absAX)
{
    for (int64_t i = 0; i < nrows; ++i) {
        for (int64_t c = 0; c < k; ++c) {
            double s = 0.0, t = 0.0;
            for (int64_t j = rowptr[i]; j < rowptr[i + 1]; ++j) {
                double a = (double)vals[j], b = (double)X[(int64_t)colidx[j] * ldx + c];
                s += a * b;
                t += fabs(a) * fabs(b);
            }
            double r = (beta == 0.0) ? alpha * s : alpha * s + beta * (double)Y0[i * ldy + c];
            Y[i * ldy + c] = (float)r;
            if (absAX) absAX[i * k + c] = t;
        }
    }
}

/* ---- Row partition reference --------------------------------------------
 * Two levels.
 *
 * (1) Stream chunks.  Rows are taken in chunks of chunk_rows consecutive rows
 * (chunk c = rows c*chunk_rows .. min((c+1)*chunk_rows, nrows) - 1).  With M
 * the largest row length in the chunk, the chunk's class is
 *   0 (not a stream chunk)  if it holds fewer than chunk_min_nnz entries or
 *                           M > 16*chunk_rows,
 *   k = 1, 2, 3, 4          otherwise, the smallest k with M <= 2^k * chunk_rows
 *                           (lane groups of 2^k lanes per row: rows up to 64,
 *                           128, 256, 512 entries for chunk_rows = 32 - the
 *                           per-chunk form of "entries per row, rounded up")
 *                           that also satisfies (entries of the chunk) <=
 *                           2^k * 16 * chunk_rows, so that the 2^(k-1)
 *                           wavefronts sharing the chunk get at most 1024
 *                           entries each on average; if no k <= 4 does, the
 *                           first condition alone decides.
 * stream_chunks lists the chunk ids class by class (class 1 first), ascending
 * inside a class; stream_offset[0..4] are the class boundaries in that list.
 *
 * (2) Bins, over the rows of all other chunks only.  Per-row lane count in the
 * spirit of the vector-length estimate of Section 4.2 (entries per row,
 * rounded up, clamped to the hardware vector width), applied row by row
 * instead of once per matrix and rounded up to a power of two, with the
 * wavefront width `wave` as the clamp:
 *   bin 0                : L == 0
 *   bin b, 1 <= b <= B-3 : smallest b with 2^(b-1) >= L, for 1 <= L <= wave
 *                          (wave = 2^(B-3))
 *   bin B-2              : wave < L <= long_threshold
 *   bin B-1              : L > long_threshold
 * With wave = 64 this gives B = 10 bins.
 */
static int bin_of_length(int64_t L, int64_t wave, int64_t long_threshold)
{
    if (L == 0) return 0;
    if (L <= wave) {
        int b = 1;
        int64_t g = 1;
        while (g < L) { g *= 2; ++b; }
        return b;
    }
    int top = 1;
    for (int64_t g = 1; g < wave; g *= 2) ++top; /* top = 1 + log2(wave) = last group bin */
    return (L <= long_threshold) ? top + 1 : top + 2;
}

/* Number of bins for a given wave width. */
int oracle_partition_num_bins(int64_t wave)
{
    return bin_of_length(wave + 1, wave, wave + 1) + 2;
}

static int chunk_class_plain(int64_t c, int64_t nrows, const int32_t *rowptr, int64_t chunk_rows,
                       int64_t chunk_min_nnz)
{
    int64_t first = c * chunk_rows;
    int64_t last = first + chunk_rows < nrows ? first + chunk_rows : nrows;
    int64_t longest = 0;
    for (int64_t i = first; i < last; ++i)
        if (rowptr[i + 1] - rowptr[i] > longest) longest = rowptr[i + 1] - rowptr[i];
    int64_t entries = rowptr[last] - rowptr[first];
    if (entries < chunk_min_nnz) return 0;
    int by_length = 0;
    for (int k = 4; k >= 1; --k)
        if (longest <= ((int64_t)1 << k) * chunk_rows) by_length = k;
    if (by_length == 0) return 0;
    for (int k = by_length; k <= 4; ++k)
        if (entries <= ((int64_t)1 << k) * 16 * chunk_rows) return k;
    return by_length;
}

/* The class a chunk finally has: a chunk listed in `demoted` (may be NULL: none) is not a stream
 * chunk whatever its rows look like (see oracle_demoted_chunks). */
static int chunk_class(int64_t c, int64_t nrows, const int32_t *rowptr, int64_t chunk_rows,
                       int64_t chunk_min_nnz, const uint8_t *demoted)
{
    if (demoted && demoted[c]) return 0;
    return chunk_class_plain(c, nrows, rowptr, chunk_rows, chunk_min_nnz);
}

/* Pass 0: stream_chunks[] (caller provides ceil(nrows/chunk_rows) slots) and
 * stream_offset[5]; returns the number of stream chunks. */
int64_t oracle_partition_stream_chunks(int64_t nrows, const int32_t *rowptr, int64_t chunk_rows,
                                       int64_t chunk_min_nnz, const uint8_t *demoted,
                                       int32_t *stream_chunks, int32_t *stream_offset)
{
    int64_t count = 0;
    int64_t nchunks = (nrows + chunk_rows - 1) / chunk_rows;
    for (int k = 1; k <= 4; ++k) {
        stream_offset[k - 1] = (int32_t)count;
        for (int64_t c = 0; c < nchunks; ++c)
            if (chunk_class(c, nrows, rowptr, chunk_rows, chunk_min_nnz, demoted) == k)
                stream_chunks[count++] = (int32_t)c;
    }
    stream_offset[4] = (int32_t)count;
    return count;
}

/* Level 1b: 16-bit column codes for the stream chunks (class >= 1).
 *  - A chunk is "narrow" if its largest and smallest column differ by at most 65535:
 *    chunk_base[c] = its smallest column, col16[j] = colidx[j] - chunk_base[c].
 *  - Otherwise, with frames of 2048 columns (frame of a column = column >> 11), a chunk whose
 *    entries touch at most 32 distinct frames is "framed": chunk_base[c] = -2,
 *    frame_table[32*c + k] = its k-th smallest frame (k below the count; the largest frame
 *    repeated above it), col16[j] = (k << 11) | (colidx[j] & 2047) with k the rank of the
 *    entry's frame.
 *  - Every other chunk: chunk_base -1, col16 0, frame_table 0.
 * counts[0] = entries in narrow chunks, counts[1] = entries in framed chunks; the compression is
 * in use when together they are at least half of all entries (and not zero).  chunk_base has
 * ceil(nrows/chunk_rows) elements, frame_table 32 times as many, col16 has rowptr[nrows]. */
static int cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

void oracle_index16(int64_t nrows, const int32_t *rowptr, const int32_t *colidx, int64_t chunk_rows,
                    int64_t chunk_min_nnz, int32_t *chunk_base, int32_t *frame_table, uint16_t *col16,
                    int32_t *scratch, int64_t *counts)
{
    int64_t nchunks = (nrows + chunk_rows - 1) / chunk_rows;
    counts[0] = counts[1] = 0;
    for (int64_t j = 0; j < rowptr[nrows]; ++j) col16[j] = 0;
    for (int64_t c = 0; c < nchunks; ++c) {
        chunk_base[c] = -1;
        for (int k = 0; k < 32; ++k) frame_table[32 * c + k] = 0;
        if (chunk_class(c, nrows, rowptr, chunk_rows, chunk_min_nnz, NULL) == 0) continue;
        int64_t last = (c + 1) * chunk_rows < nrows ? (c + 1) * chunk_rows : nrows;
        int64_t b = rowptr[c * chunk_rows], e = rowptr[last];
        int32_t lo = colidx[b], hi = colidx[b];
        for (int64_t j = b; j < e; ++j) {
            if (colidx[j] < lo) lo = colidx[j];
            if (colidx[j] > hi) hi = colidx[j];
        }
        if ((int64_t)hi - lo <= 65535) {
            chunk_base[c] = lo;
            for (int64_t j = b; j < e; ++j) col16[j] = (uint16_t)(colidx[j] - lo);
            counts[0] += e - b;
            continue;
        }
        /* distinct frames, ascending (scratch holds one int per entry of the chunk) */
        for (int64_t j = b; j < e; ++j) scratch[j - b] = colidx[j] >> 11;
        qsort(scratch, (size_t)(e - b), sizeof(int32_t), cmp_i32);
        int64_t distinct = 0;
        for (int64_t i = 0; i < e - b; ++i)
            if (i == 0 || scratch[i] != scratch[i - 1]) scratch[distinct++] = scratch[i];
        if (distinct > 32) continue;
        chunk_base[c] = -2;
        for (int k = 0; k < 32; ++k)
            frame_table[32 * c + k] = scratch[k < distinct ? k : distinct - 1];
        for (int64_t j = b; j < e; ++j) {
            int k = 0;
            while (frame_table[32 * c + k] != (colidx[j] >> 11)) ++k;
            col16[j] = (uint16_t)((k << 11) | (colidx[j] & 2047));
        }
        counts[1] += e - b;
    }
}

/* When x is far larger than a level-2 cache (the caller checks that: the column split's own
 * condition), a chunk that would stream although its columns are neither narrow nor framed
 * (chunk_base[c] == -1 from oracle_index16) and that has a row of more than `wave` entries is
 * demoted: its rows go to the bins, where the column split orders their gathers.
 * demoted[c] = 1 for those chunks, 0 otherwise. */
void oracle_demoted_chunks(int64_t nrows, const int32_t *rowptr, int64_t chunk_rows, int64_t chunk_min_nnz,
                           int64_t wave, const int32_t *chunk_base, uint8_t *demoted)
{
    int64_t nchunks = (nrows + chunk_rows - 1) / chunk_rows;
    for (int64_t c = 0; c < nchunks; ++c) {
        demoted[c] = 0;
        if (chunk_class_plain(c, nrows, rowptr, chunk_rows, chunk_min_nnz) == 0 || chunk_base[c] != -1) continue;
        int64_t last = (c + 1) * chunk_rows < nrows ? (c + 1) * chunk_rows : nrows;
        for (int64_t i = c * chunk_rows; i < last; ++i)
            if (rowptr[i + 1] - rowptr[i] > wave) demoted[c] = 1;
    }
}

/* Level 1c: row patterns of the stream chunks (final class >= 1).
 * The list of a non-empty row i is its diagonals colidx[j] - i in stored order; its SHAPE is the
 * same list minus its first element.  Going through the rows of a chunk in ascending order, a
 * row takes the first stored list (in order of insertion) that has its length and its shape and
 * whose shift = (the row's first diagonal) - (the stored list's first diagonal) lies in
 * [-64, 63]; a row for which no stored list qualifies appends its own list to the chunk's table
 * (shift 0).
 * row_pat[i] = (where the taken list starts in the table) | ((shift & 127) << 9), 0 for empty
 * rows.  Rows of a regular grid all have one list and shift 0; the rows of the unknowns of one
 * grid point in a matrix with several unknowns per point hold the same columns, so their lists
 * are one shape with shifts 0, -1, -2, ...
 * A chunk is "patterned" when no row has more than max_row entries, at most max_patterns lists
 * were stored, the table has at most max_table (<= 512) diagonals and twice the table length
 * does not exceed the chunk's entry count; otherwise its
 * table is empty and row_pat is 0 for its rows.
 * pat_off[0 .. nchunks] = exclusive scan of the table lengths (pat_off[c+1] == pat_off[c] for
 * chunks without patterns); pool (may be NULL to get the sizes only) receives the tables back
 * to back.  *entries = number of matrix entries in patterned chunks.
 * Reconstruction: colidx[rowptr[i] + k] == i + shift_i + pool[pat_off[c] + (row_pat[i] & 511) + k]. */
void oracle_row_patterns(int64_t nrows, const int32_t *rowptr, const int32_t *colidx, int64_t chunk_rows,
                         int64_t chunk_min_nnz, const uint8_t *demoted, int64_t max_row, int64_t max_patterns,
                         int64_t max_table, int32_t *pat_off, uint16_t *row_pat, int32_t *pool,
                         int64_t *entries)
{
    int64_t nchunks = (nrows + chunk_rows - 1) / chunk_rows;
    int32_t table[4096];
    int64_t start[64], length[64];
    *entries = 0;
    pat_off[0] = 0;
    for (int64_t i = 0; i < nrows; ++i) row_pat[i] = 0;
    for (int64_t c = 0; c < nchunks; ++c) {
        pat_off[c + 1] = pat_off[c];
        if (chunk_class(c, nrows, rowptr, chunk_rows, chunk_min_nnz, demoted) == 0) continue;
        int64_t first = c * chunk_rows;
        int64_t last = first + chunk_rows < nrows ? first + chunk_rows : nrows;
        int64_t P = 0, L = 0;
        int ok = 1;
        for (int64_t i = first; i < last && ok; ++i) {
            int64_t b = rowptr[i], len = rowptr[i + 1] - b;
            if (len == 0) continue;
            if (len > max_row) { ok = 0; break; }
            int64_t found = -1;
            for (int64_t p = 0; p < P && found < 0; ++p) {
                if (length[p] != len) continue;
                int64_t shift = ((int64_t)colidx[b] - i) - table[start[p]];
                if (shift < -64 || shift > 63) continue;    /* too far away to be coded: not a match */
                int same = 1;
                for (int64_t k = 0; k < len; ++k)          /* shapes: differences from the first element */
                    if ((int64_t)table[start[p] + k] - table[start[p]] != (int64_t)colidx[b + k] - colidx[b]) same = 0;
                if (same) found = p;
            }
            if (found < 0) {
                if (P == max_patterns || L + len > max_table) { ok = 0; break; }
                start[P] = L;
                length[P] = len;
                for (int64_t k = 0; k < len; ++k) table[L + k] = colidx[b + k] - (int32_t)i;
                found = P++;
                L += len;
            }
            int64_t shift = ((int64_t)colidx[b] - i) - table[start[found]];
            row_pat[i] = (uint16_t)(start[found] | ((shift & 127) << 9));
        }
        int64_t chunk_entries = rowptr[last] - rowptr[first];
        if (!ok || 2 * L > chunk_entries) {
            for (int64_t i = first; i < last; ++i) row_pat[i] = 0;
            continue;
        }
        if (pool)
            for (int64_t t = 0; t < L; ++t) pool[pat_off[c] + t] = table[t];
        pat_off[c + 1] = pat_off[c] + (int32_t)L;
        *entries += chunk_entries;
    }
}

/* Pass 1: bin_offset[num_bins+1] (exclusive scan of per-bin row counts) and
 * row_perm[] (ids of the rows outside stream chunks, grouped by bin, ascending
 * inside each bin; bin_offset[num_bins] of them).  Returns through *num_long
 * the number of rows in the last bin and through *num_tiles the number of
 * tiles T = ceil(total long nnz / tile_nnz). */
void oracle_partition_rows(int64_t nrows, const int32_t *rowptr, int64_t wave,
                           int64_t long_threshold, int64_t tile_nnz, int64_t chunk_rows,
                           int64_t chunk_min_nnz, const uint8_t *demoted, int32_t *bin_offset, int32_t *row_perm,
                           int64_t *num_long, int64_t *num_tiles)
{
    int nb = oracle_partition_num_bins(wave);
    for (int b = 0; b <= nb; ++b) bin_offset[b] = 0;
    for (int64_t i = 0; i < nrows; ++i) {
        if (chunk_class(i / chunk_rows, nrows, rowptr, chunk_rows, chunk_min_nnz, demoted)) continue;
        bin_offset[bin_of_length(rowptr[i + 1] - rowptr[i], wave, long_threshold) + 1] += 1;
    }
    for (int b = 0; b < nb; ++b) bin_offset[b + 1] += bin_offset[b];
    int64_t long_nnz = 0;
    for (int b = 0; b < nb; ++b) {
        int64_t at = bin_offset[b];
        for (int64_t i = 0; i < nrows; ++i) {
            int64_t L = rowptr[i + 1] - rowptr[i];
            if (chunk_class(i / chunk_rows, nrows, rowptr, chunk_rows, chunk_min_nnz, demoted)) continue;
            if (bin_of_length(L, wave, long_threshold) != b) continue;
            row_perm[at++] = (int32_t)i;
            if (b == nb - 1) long_nnz += L;
        }
    }
    *num_long = bin_offset[nb] - bin_offset[nb - 1];
    *num_tiles = (long_nnz + tile_nnz - 1) / tile_nnz;
}

/* Pass 2, over the rows of the last bin in row_perm order:
 *   long_off[0..m]  exclusive scan of their lengths (their entries laid end
 *                   to end form the "long nnz space" of size long_off[m]);
 *   tile t covers long nnz positions [t*tile_nnz, (t+1)*tile_nnz);
 *   tile_row[t]     index r in 0..m-1 of the long row holding position
 *                   t*tile_nnz, i.e. the largest r with long_off[r] <= t*tile_nnz;
 *   tile_nz[t]      t*tile_nnz - long_off[tile_row[t]], the offset inside it;
 *   sentinel        tile_row[T] = m, tile_nz[T] = 0.
 */
void oracle_partition_tiles(const int32_t *rowptr, int64_t tile_nnz, const int32_t *long_rows,
                            int64_t m, int64_t T, int32_t *long_off, int32_t *tile_row,
                            int32_t *tile_nz)
{
    long_off[0] = 0;
    for (int64_t r = 0; r < m; ++r)
        long_off[r + 1] = long_off[r] + (rowptr[long_rows[r] + 1] - rowptr[long_rows[r]]);
    for (int64_t t = 0; t < T; ++t) {
        int64_t pos = t * tile_nnz;
        int64_t r = 0;
        while (r + 1 <= m - 1 && long_off[r + 1] <= pos) ++r;
        tile_row[t] = (int32_t)r;
        tile_nz[t] = (int32_t)(pos - long_off[r]);
    }
    tile_row[T] = (int32_t)m;
    tile_nz[T] = 0;
}

/* ---- Column split of the rows with more than `wave` entries ---------------
 * When x is much larger than a level-2 cache, the rows of the last two bins
 * (split_rows[0..S-1], in row_perm order) are cut at the column-block
 * boundaries b*W, b = 0..nb: cut[b*S + r] is the first entry j of row
 * split_rows[r] with colidx[j] >= b*W (so cut[0*S + r] = rowptr[row] and
 * cut[nb*S + r] = rowptr[row+1]).  Virtual row v = b*S + r owns the entries
 * cut[v] .. cut[v + S] - 1.  The cut is only meaningful when every split row
 * has non-decreasing columns; *sorted reports that.
 */
void oracle_split_cuts(const int32_t *rowptr, const int32_t *colidx, const int32_t *split_rows,
                       int64_t S, int64_t nb, int64_t W, int32_t *cut, int32_t *sorted)
{
    *sorted = 1;
    for (int64_t r = 0; r < S; ++r) {
        int64_t rb = rowptr[split_rows[r]], re = rowptr[split_rows[r] + 1];
        for (int64_t j = rb; j + 1 < re; ++j)
            if (colidx[j] > colidx[j + 1]) *sorted = 0;
        int64_t j = rb;
        for (int64_t b = 0; b <= nb; ++b) {
            while (j < re && (int64_t)colidx[j] < b * W) ++j;
            cut[b * S + r] = (int32_t)(b == nb ? re : j);
        }
    }
}
