/*
 * lapis.h - C ABI of the MI355X (gfx950) CSR SpMV / SpMM library.
 *
 * The library computes the sparse kernel the LAPIS paper generates and times in
 * Section 6.2: y := A x with A in compressed sparse row form and x, y dense,
 * extended BLAS-style to y = alpha*A*x + beta*y, and its multi-vector form
 * Y = alpha*A*X + beta*Y.  The row / entry traversal is the CSR loop nest of
 * Section 4.2 ("Parallelism estimation"): row i owns the entries
 * offsets[i] .. offsets[i+1]-1 of the value and column-index arrays.
 *
 * Conventions (after Section 5, where the generated code is wrapped in
 * unmangled functions taking raw pointers and sizes, and Section 4.3, where
 * data stays on the device between kernels):
 *   - every array argument is a DEVICE pointer unless its name starts with h_;
 *   - the library never copies, frees or writes the caller's matrix arrays;
 *   - every function returns a status code, never throws, aborts or prints;
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).
 *
 * Row indices and column indices are 32-bit; nrows+1 must fit in int32 and nnz must not
 * exceed LAPIS_MAX_NNZ.
 */
#ifndef LAPIS_H
#define LAPIS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- status codes ------------------------------------------------------- */
#define LAPIS_OK               0
#define LAPIS_ERR_INVALID_ARG  1   /* null pointer, negative size, size beyond int32, ld < k, k <= 0 */
#define LAPIS_ERR_UNSUPPORTED  2   /* dtype not LAPIS_F32 / LAPIS_F64 */
#define LAPIS_ERR_ALLOC        3   /* device or host allocation failed */
#define LAPIS_ERR_DEVICE       4   /* a HIP call failed; text via lapis_last_error() */

/* ---- value types -------------------------------------------------------- */
#define LAPIS_F32 0
#define LAPIS_F64 1

/* ---- row partition constants ---------------------------------------------
 * The levels of the analysis pass.
 *
 * Level 1, stream chunks.  Rows are taken in chunks of LAPIS_STREAM_ROWS
 * consecutive rows (chunk c = rows c*LAPIS_STREAM_ROWS ...).  With M the longest
 * row of the chunk, its class is 0 (not a stream chunk) if the chunk holds fewer
 * than LAPIS_STREAM_MIN_NNZ entries or M > 16*LAPIS_STREAM_ROWS, else the
 * smallest k in 1..4 with M <= 2^k * LAPIS_STREAM_ROWS (groups of 2^k lanes per
 * row, rows up to 64 / 128 / 256 / 512 entries - the per-chunk form of the
 * estimate of Section 4.2, entries per row, rounded up) and with at most
 * 2^k * 16 * LAPIS_STREAM_ROWS entries in the chunk (so each of the 2^(k-1)
 * wavefronts sharing it gets about one LDS window); if no k <= 4 meets the
 * second condition, the first alone decides.  A stream chunk's
 * entries are one contiguous piece of the value / column arrays, which
 * wavefronts stream through LDS.  If d_colidx or d_vals is not 16-byte aligned,
 * no chunk is a stream chunk.
 *
 * Level 2, bins, for the rows of all other chunks.  It generalises the
 * vector-length estimate of Section 4.2 (entries per row, rounded up, clamped
 * to the hardware vector width) from one value per matrix to one value per row.
 * With L the number of entries of a row:
 *   bin 0      L == 0
 *   bin b      1 <= b <= 7: smallest b with 2^(b-1) >= L   (1 <= L <= 64);
 *              2^(b-1) is the row's lane-group size, 64 = the gfx950 wavefront
 *   bin 8      64 < L <= LAPIS_LONG_THRESHOLD  (one wavefront walks the row)
 *   bin 9      L > LAPIS_LONG_THRESHOLD        (row is cut into tiles)
 * The entries of the bin-9 rows, laid end to end in row order, are cut into
 * tiles of LAPIS_TILE_NNZ entries; LAPIS_LONG_THRESHOLD >= LAPIS_TILE_NNZ, so a
 * tile touches at most two rows.
 *
 * Demotion: when x is far larger than a level-2 cache (nb >= 2 in level 3 below), a chunk
 * that would stream but whose columns are neither narrow nor framed (see
 * lapis_csr_copy_index16) and that has a row of more than LAPIS_WAVE entries does not stream:
 * its rows are binned like those of any class-0 chunk.
 *
 * Level 3, column split (lapis_spmv only), for the rows of bins 8 and 9 when x
 * is far larger than a level-2 cache.  With e the size of a value in bytes:
 * nb = min(LAPIS_SPLIT_MAX_BLOCKS, ceil(ncols / (LAPIS_SPLIT_BLOCK_BYTES / e)))
 * column blocks of width W = ceil(ncols / nb); the split is off when nb < 2,
 * when bins 8 and 9 are empty, or when one of their rows has decreasing
 * columns.  Let split_rows[0..S-1] be the rows of bins 8 and 9 with at most
 * LAPIS_HUGE_ROW entries, in row_perm order (the longer ones: level 3b below).
 * cut[b*S + r] is the first entry of row split_rows[r] whose column is
 * >= b*W (b = 0..nb; cut[nb*S + r] is the row's end).  Virtual row v = b*S + r
 * owns the entries cut[v] .. cut[v+S]-1; the virtual rows are binned and tiled
 * by the level-2 rule (no stream chunks), processed block after block so that
 * the gathers of one column block stay cache resident, and each split row's nb
 * partial sums are added in ascending block order.
 *
 * Level 3b, for the rows of more than LAPIS_HUGE_ROW entries when the split is on:
 * huge_rows[0..H-1] are those rows in row_perm order (all in bin 9, so ascending).  They are
 * cut at column blocks that hold LAPIS_LDS_BLOCK_BYTES of x: nbf = ceil(ncols / Wf) blocks of
 * Wf = LAPIS_LDS_BLOCK_BYTES / e columns; fcut[b*H + h] is the first entry of row huge_rows[h]
 * whose column is >= b*Wf (b = 0..nbf; fcut[nbf*H + h] is the row's end).  A workgroup keeps
 * one block of x in LDS while the pieces of all huge rows in that block stream by.  The split
 * is also off when (nb+1)*S or (nbf+1)*H exceeds int32.
 */
#define LAPIS_NUM_BINS        10
#define LAPIS_WAVE            64
#define LAPIS_LONG_THRESHOLD  4096
#define LAPIS_TILE_NNZ        4096
#define LAPIS_STREAM_ROWS     32
#define LAPIS_STREAM_MIN_NNZ  64
#define LAPIS_SPLIT_BLOCK_BYTES 2097152   /* 2 MiB of x per column block */
#define LAPIS_MAX_NNZ 2147418112        /* 2^31 - 2^16: entry ids plus a tile stay inside int32 */
#define LAPIS_SPLIT_MAX_BLOCKS  32
#define LAPIS_HUGE_ROW 16384             /* rows with more entries are cut at LDS-sized column blocks */
#define LAPIS_LDS_BLOCK_BYTES 65536      /* bytes of x one such block holds */
#define LAPIS_PATTERN_MAX_ROW 128        /* longest row a patterned chunk may have (lapis_csr_copy_patterns) */
#define LAPIS_PATTERN_SLOTS 8            /* distinct row patterns per chunk at most */
#define LAPIS_PATTERN_TABLE 512          /* diagonals in a chunk's pattern table at most */

typedef struct lapis_csr lapis_csr_t;   /* opaque handle */

/*
 * lapis_csr_create - wrap a device-resident CSR matrix and run the row
 * partition analysis (the per-row form of the Section 4.2 estimate) on it.
 *
 *   out        receives the handle; set to NULL on any error
 *   nrows, ncols, nnz   sizes, all >= 0; nrows+1 must fit in int32, nnz <= LAPIS_MAX_NNZ
 *   d_rowptr   int32[nrows+1], d_rowptr[0] == 0, non-decreasing,
 *              d_rowptr[nrows] == nnz
 *   d_colidx   int32[nnz], 0 <= d_colidx[j] < ncols; columns inside a row need
 *              be neither sorted nor distinct (repeated columns add up)
 *   d_vals     float[nnz] or double[nnz] according to dtype
 *   dtype      LAPIS_F32 or LAPIS_F64; x, y, X, Y of later calls have this type
 *   hip_stream stream the analysis kernels run on
 *
 * Ownership: the three arrays are BORROWED; they must stay allocated and
 * unchanged until lapis_csr_destroy.  The handle owns only its analysis
 * buffers (stream chunk list, bin offsets, per-bin row lists, tile table,
 * per-tile partial sums).
 * The call synchronises hip_stream (it reads back the bin counts and checks
 * d_rowptr[0] == 0 and d_rowptr[nrows] == nnz; a mismatch is
 * LAPIS_ERR_INVALID_ARG).  d_colidx and d_vals may be NULL when nnz == 0.
 */
int lapis_csr_create(lapis_csr_t **out, int64_t nrows, int64_t ncols, int64_t nnz,
                     const int32_t *d_rowptr, const int32_t *d_colidx, const void *d_vals,
                     int dtype, void *hip_stream);

/*
 * lapis_spmv - y = alpha*A*x + beta*y  (Section 6.2: y := A x; alpha = 1, beta = 0).
 *
 *   d_x   ncols elements of A's dtype, contiguous
 *   d_y   nrows elements of A's dtype, contiguous; must not overlap d_x or A
 *   alpha, beta   passed as double; rounded to float for LAPIS_F32 matrices
 *
 * beta == 0 makes d_y write-only: its old contents (NaN included) are ignored.
 * Rows without entries receive beta*y (exactly +0 when beta == 0).
 * Asynchronous: the kernels are enqueued on hip_stream and the call returns;
 * no allocation, no host-device copy, no host synchronisation.  Matrices with rows
 * in bin 9 or with a column split use scratch owned by the handle (per-tile and
 * per-virtual-row sums).  Calls on one handle from different streams are therefore
 * ordered by the library: every such product records an event on its stream, and a
 * product enqueued on another stream than the previous one first makes its stream wait
 * for that event (the products of one handle run one after the other, whatever their
 * streams; handles without scratch - no bin-9 row, no split - are not ordered and may
 * overlap freely).  The one exception is a stream that is being captured into a HIP
 * graph: nothing is recorded or waited for there, and the caller must not let a captured
 * product of such a handle overlap another product of the same handle.
 */
int lapis_spmv(const lapis_csr_t *A, double alpha, const void *d_x, double beta, void *d_y,
               void *hip_stream);

/*
 * lapis_spmv_static_scratch - lapis_spmv for callers that must not allocate and cannot rely on
 * memory the handle allocated: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, result, dtype, beta == 0 and asynchrony rules as lapis_spmv
 * and the same kernels; the intermediate sums (per-tile sums of rows in bin 9, per-virtual-row
 * sums of the column split, per-block sums of the rows above LAPIS_HUGE_ROW entries) go to a
 * buffer of LAPIS_STATIC_SCRATCH_BYTES that is part of the library's code object instead of the
 * handle's own buffers.  Every GPU the library runs on holds one copy of that buffer until the
 * process ends; its address is looked up once per device, on the first call made with that
 * device current.  The call itself allocates nothing, frees nothing and copies nothing.
 * Nothing in the buffer has to be cleared between calls: every sum a call reads it has written
 * before.  ALL calls on one GPU share the buffer, whatever their handle or stream: two calls
 * that overlap in time on one GPU race and give wrong results; order them on one stream or
 * with events.
 * lapis_spmv_scratch_bytes(A) is what a product with A needs (0 for matrices without such rows;
 * -1 for a NULL handle).  A matrix that needs more than LAPIS_STATIC_SCRATCH_BYTES is refused
 * with LAPIS_ERR_INVALID_ARG and a message that names both numbers; nothing is launched then.
 */
#define LAPIS_STATIC_SCRATCH_BYTES 33554432   /* 32 MiB */
int64_t lapis_spmv_scratch_bytes(const lapis_csr_t *A);
int lapis_spmv_static_scratch(const lapis_csr_t *A, double alpha, const void *d_x, double beta, void *d_y,
                              void *hip_stream);

/*
 * lapis_spmv_transpose - y = alpha*A^T*x + beta*y from the CSR arrays of A: the column-wise
 * (CSC) traversal of the sparse loop pattern of Section 4.2 (the CSR arrays of A are the CSC
 * arrays of A^T; equivalently, the product of a CSC-stored matrix with a vector).
 *
 *   d_x   nrows elements of A's dtype, contiguous
 *   d_y   ncols elements of A's dtype, contiguous; must not overlap d_x or A
 *
 * beta == 0 makes d_y write-only; columns without entries receive beta*y.  The sums are formed
 * by floating-point atomic additions in memory, in no fixed order: each element lies within
 * the rounding bound of a serial evaluation, but two calls may differ in the last bits.
 * Asynchronous on hip_stream; no allocation, copy or synchronisation; uses no scratch of the
 * handle.
 */
int lapis_spmv_transpose(const lapis_csr_t *A, double alpha, const void *d_x, double beta, void *d_y,
                         void *hip_stream);

/*
 * lapis_csr_create_transpose - a handle for A^T (ncols x nrows) built on the device from the
 * arrays of A as they are at the time of the call: the explicit form of the column-wise
 * traversal of Section 4.2, for callers that apply A^T many times.  lapis_spmv / lapis_spmm on
 * the new handle compute A^T x / A^T X with the same kernels and the same analysis as for any
 * other matrix, with a fixed order of additions.
 *
 * The new handle OWNS its CSR arrays (device memory allocated here: (ncols+1 + nnz) int32 and
 * nnz values, plus 8*nnz + 4*ncols bytes of temporaries during the call) and does not refer to
 * A afterwards; later changes to A's values are not followed.  Inside row c of A^T the entries
 * are ordered by (row of A, position inside that row), duplicates kept: the result of a serial
 * row-by-row transposition, unique, so it can be compared bit for bit.
 * Synchronises hip_stream.  Destroy with lapis_csr_destroy.
 *
 * lapis_csr_shape reports a handle's sizes and dtype (any out pointer may be NULL).
 * lapis_csr_copy_arrays copies a handle's CSR arrays (borrowed or owned) to HOST buffers of
 * nrows+1, nnz and nnz elements (any may be NULL); it synchronises the device.
 */
int lapis_csr_create_transpose(lapis_csr_t **out, const lapis_csr_t *A, void *hip_stream);
int lapis_csr_shape(const lapis_csr_t *A, int64_t *nrows, int64_t *ncols, int64_t *nnz, int *dtype);
int lapis_csr_copy_arrays(const lapis_csr_t *A, int32_t *h_rowptr, int32_t *h_colidx, void *h_vals);

/*
 * lapis_spmv_paper_shape - the same product as lapis_spmv, computed with the
 * kernel shape the paper's loop mapping generates (Section 4.2): one vector
 * length for the whole matrix, g = the average number of entries per row
 * rounded up ("Parallelism estimation": (k+N-1)/N with k = offsets[N]), clamped
 * to the back end's maximum (the 64-lane wavefront here; the paper names 32 for
 * CUDA) and rounded up to a power of two; g lanes stride each row, their sums
 * are reduced and one lane stores y[i].  It ignores the row partition.  It
 * exists to put the paper's method beside the tuned kernels on the same
 * hardware.  Arguments, dtype, beta == 0 and asynchrony rules as lapis_spmv.
 */
int lapis_spmv_paper_shape(const lapis_csr_t *A, double alpha, const void *d_x, double beta,
                           void *d_y, void *hip_stream);

/* The vector length lapis_spmv_paper_shape uses: (nnz + nrows - 1) / nrows (Section 4.2,
 * "Parallelism estimation"), clamped to LAPIS_WAVE and rounded up to a power of two; 1 for an
 * empty matrix.  Host-only, no device access. */
int lapis_paper_vector_length(int64_t nrows, int64_t nnz);

/*
 * lapis_spmm - Y = alpha*A*X + beta*Y for k right-hand sides; column c of Y is
 * by definition lapis_spmv applied to column c of X (the paper times only the
 * single-vector product; this is its multi-vector form).
 *
 *   d_X   ncols x k, ROW-MAJOR, leading dimension ldx >= k (in elements)
 *   d_Y   nrows x k, ROW-MAJOR, leading dimension ldy >= k; must not overlap d_X or A
 *   k     >= 1
 *
 * Same dtype, beta == 0, asynchrony and concurrency rules as lapis_spmv.
 */
int lapis_spmm(const lapis_csr_t *A, int64_t k, double alpha, const void *d_X, int64_t ldx,
               double beta, void *d_Y, int64_t ldy, void *hip_stream);

/*
 * lapis_csr_destroy - free the handle's own buffers.  NULL is a no-op that
 * returns LAPIS_OK.  The caller must have synchronised every stream that still
 * has work using the handle.  The borrowed matrix arrays are left alone.
 */
int lapis_csr_destroy(lapis_csr_t *A);

/* ---- inspection of the row partition (for bit-exact checks) --------------
 * lapis_csr_partition_sizes: *num_stream = number of stream chunks,
 * *num_binned = number of rows outside stream chunks (the length of row_perm),
 * *num_long = rows in bin 9, *num_tiles = number of tiles T.  Any pointer may
 * be NULL.
 * lapis_csr_copy_partition: copies to HOST buffers the caller owns (any may be
 * NULL to skip it):
 *   h_stream_chunks int32[num_stream]     stream chunk ids, class 1 first, ascending in a class
 *   h_stream_offset int32[5]              class boundaries in h_stream_chunks
 *   h_bin_offset int32[LAPIS_NUM_BINS+1]  exclusive scan of per-bin row counts
 *   h_row_perm   int32[num_binned]        row ids grouped by bin, ascending in each bin
 *   h_long_off   int32[num_long+1]        exclusive scan of the bin-9 rows' lengths
 *   h_tile_row   int32[T+1]               bin-9 row (index into its list) holding
 *                                         long position t*LAPIS_TILE_NNZ; [T] = num_long
 *   h_tile_nz    int32[T+1]               offset of that position inside the row; [T] = 0
 * Synchronises the device.
 */
int lapis_csr_partition_sizes(const lapis_csr_t *A, int64_t *num_stream, int64_t *num_binned,
                              int64_t *num_long, int64_t *num_tiles);
int lapis_csr_copy_partition(const lapis_csr_t *A, int32_t *h_stream_chunks, int32_t *h_stream_offset,
                             int32_t *h_bin_offset, int32_t *h_row_perm, int32_t *h_long_off,
                             int32_t *h_tile_row, int32_t *h_tile_nz);

/* The column split (level 3).  lapis_csr_split_sizes: *num_blocks = nb (0: the split is off),
 * *block_width = W, *num_split_rows = S, and for the virtual rows *num_binned (= nb*S),
 * *num_long, *num_tiles as in lapis_csr_partition_sizes.  lapis_csr_copy_split copies to HOST
 * buffers (any may be NULL): h_cut int32[(nb+1)*S] and the bins / row lists / tile table of the
 * virtual rows, laid out as in lapis_csr_copy_partition.  It returns LAPIS_ERR_INVALID_ARG when
 * the split is off.  Synchronises the device. */
int lapis_csr_split_sizes(const lapis_csr_t *A, int64_t *num_blocks, int64_t *block_width,
                          int64_t *num_split_rows, int64_t *num_binned, int64_t *num_long,
                          int64_t *num_tiles);
int lapis_csr_copy_split(const lapis_csr_t *A, int32_t *h_cut, int32_t *h_bin_offset,
                         int32_t *h_row_perm, int32_t *h_long_off, int32_t *h_tile_row,
                         int32_t *h_tile_nz);

/* Level 3b.  lapis_csr_huge_sizes: *num_huge = H, *num_fblocks = nbf, *fblock_width = Wf (all 0
 * when the split is off).  lapis_csr_copy_huge copies to HOST buffers (any may be NULL):
 * h_split_rows int32[S], h_huge_rows int32[H], h_fcut int32[(nbf+1)*H]; LAPIS_ERR_INVALID_ARG
 * when the split is off.  Synchronises the device. */
int lapis_csr_huge_sizes(const lapis_csr_t *A, int64_t *num_huge, int64_t *num_fblocks, int64_t *fblock_width);
int lapis_csr_copy_huge(const lapis_csr_t *A, int32_t *h_split_rows, int32_t *h_huge_rows, int32_t *h_fcut);

/*
 * lapis_csr_copy_index16 - the 16-bit column codes the analysis builds so that the stream
 * kernels read 2 instead of 4 bytes of index per entry (an implementation choice of this
 * library, not of the paper; exposed so that it can be compared bit for bit with a CPU
 * reference).  For a stream chunk c:
 *   narrow  (largest - smallest column <= 65535): chunk_base[c] = its smallest column,
 *           col16[j] = colidx[j] - chunk_base[c];
 *   framed  (not narrow, entries in at most 32 distinct frames; frame = column >> 11):
 *           chunk_base[c] = -2, frame_table[32*c + k] = k-th smallest frame (the largest one
 *           repeated above the count), col16[j] = (rank of the entry's frame << 11) |
 *           (colidx[j] & 2047);
 *   otherwise chunk_base[c] = -1, col16 0, frame_table 0 (also for chunks that do not stream).
 * The structure is kept (*enabled = 1) only if narrow and framed chunks together hold at least
 * half of the matrix's entries; *narrow_entries and *framed_entries are those counts either way.
 *   h_chunk_base  HOST int32[C], C = ceil(nrows / LAPIS_STREAM_ROWS)
 *   h_frame_table HOST int32[32*C]        h_col16  HOST uint16[nnz]
 * The arrays are written only when *enabled is 1; any pointer may be NULL.  Synchronises the device.
 */
int lapis_csr_copy_index16(const lapis_csr_t *A, int *enabled, int64_t *narrow_entries, int64_t *framed_entries,
                           int32_t *h_chunk_base, int32_t *h_frame_table, uint16_t *h_col16);

/*
 * lapis_csr_copy_patterns - the row patterns the analysis finds in the stream chunks (an
 * implementation choice of this library, not of the paper; exposed so that it can be compared
 * bit for bit with a CPU reference).  Matrices of regular grids repeat the same list of
 * diagonals (column - row, in stored order) row after row; where the rows of a chunk share a
 * few such lists, lapis_spmv reads no column index per entry at all for that chunk.
 * For a stream chunk c (after the demotion above), going through its rows in ascending order:
 * the list of a row is its diagonals in stored order, its shape that list minus its first
 * element.  A row takes the first list stored so far (in order of insertion) that has its
 * length and its shape and whose first diagonal differs from the row's by a shift in [-64, 63]
 * (shift = the row's first diagonal - the stored one); a row that finds none appends its own
 * list to the chunk's table (shift 0).  row_pat[i] = (where the taken list starts in the table)
 * | ((shift & 127) << 9), 0 for empty rows.  Rows of a regular grid repeat one list with shift
 * 0; the rows of the unknowns of one grid point (several unknowns per point) hold the same
 * columns and share one stored list with shifts 0, -1, -2, ...  The chunk is patterned if no
 * row has more than LAPIS_PATTERN_MAX_ROW entries, at most LAPIS_PATTERN_SLOTS lists were
 * stored, the table has at most LAPIS_PATTERN_TABLE diagonals and twice its length does not
 * exceed the chunk's entries; otherwise its table is empty and row_pat is 0 for its rows.
 * pat_off[0..C] (C = ceil(nrows / LAPIS_STREAM_ROWS)) is the exclusive scan of the table lengths
 * and pool holds the tables back to back, so that for a row i of a patterned chunk c, with
 * start = row_pat[i] & 511 and shift = bits 9..15 of row_pat[i] as a signed number,
 *   colidx[rowptr[i] + k] == i + shift + pool[pat_off[c] + start + k].
 * The structure is kept (*enabled = 1) only if the patterned chunks hold at least half of the
 * matrix's entries; *pattern_entries is that count and *pool_size = pat_off[C] either way.
 *   h_pat_off HOST int32[C + 1]    h_row_pat HOST uint16[nrows]    h_pool HOST int32[*pool_size]
 * The arrays are written only when *enabled is 1; any pointer may be NULL (call once for
 * *pool_size, then again with the buffers).  Synchronises the device.
 */
int lapis_csr_copy_patterns(const lapis_csr_t *A, int *enabled, int64_t *pattern_entries, int64_t *pool_size,
                            int32_t *h_pat_off, uint16_t *h_row_pat, int32_t *h_pool);

/*
 * lapis_csr_copy_share_classes - how lapis_spmm treats each stream chunk (an implementation choice of
 * this library, exposed for comparison with a CPU reference).  On grid matrices neighbouring rows
 * need neighbouring rows of X; chunks whose rows say so through their row patterns get kernels that
 * load a row of X once for several matrix rows.  h_class[c], c < C = ceil(nrows / LAPIS_STREAM_ROWS):
 *   0  c is not a stream chunk;   LAPIS_SHARE_NONE  a stream chunk without such sharing;
 *   LAPIS_SHARE_PLAIN, LAPIS_SHARE_BLOCK3, LAPIS_SHARE_BLOCK2 as follows.
 * Of a patterned chunk take the lengths of its 32 rows (0 past the end of the matrix) and, of the first
 * row of the greatest length L, the stored list it uses (its start in the chunk's table) and its shift:
 * the reference.  A row is regular if it has length L and the reference's start - and, for PLAIN, the
 * reference's shift.  The chunk qualifies if L > 0, the stored list ascends strictly and at most
 * LAPIS_SHARE_MAX_ODD rows of the matrix in it are not regular.
 *   PLAIN: it qualifies with shifts compared, L <= 64, and (last entry of the chunk) - (its first entry
 *     rounded down to a multiple of 8) + 64 <= 1024;
 *   otherwise BLOCK3 or BLOCK2: it qualifies with shifts ignored, L <= 128, and with v = (row's place in
 *     the chunk) + (its shift), the regular rows of every aligned group of four rows have v equal to the
 *     group's least v or to that plus D, with the same D = 3 (BLOCK3) or 2 (BLOCK2) in the whole chunk and
 *     at least one row at D (rows of grid points with three or two unknowns each).
 * *enabled = 1 if the classes were computed (row patterns enabled and at least one stream chunk), else
 * h_class is left alone.  h_class HOST int32[C], may be NULL.  Synchronises the device.
 */
#define LAPIS_SHARE_PLAIN   1
#define LAPIS_SHARE_NONE    2
#define LAPIS_SHARE_BLOCK3  3
#define LAPIS_SHARE_BLOCK2  4
#define LAPIS_SHARE_MAX_ODD 4
int lapis_csr_copy_share_classes(const lapis_csr_t *A, int *enabled, int32_t *h_class);

/* max |column - row| over the matrix's entries, found by lapis_csr_create; lapis_spmm uses it to
 * decide how workgroups are dealt to the 8 XCDs (band-wide windows of X rows that overflow one
 * L2 are shared by all 8). */
int lapis_csr_half_bandwidth(const lapis_csr_t *A, int64_t *half_bandwidth);

/* The partition constants compiled into the library, in the order
 * {LAPIS_NUM_BINS, LAPIS_WAVE, LAPIS_LONG_THRESHOLD, LAPIS_TILE_NNZ,
 *  LAPIS_STREAM_ROWS, LAPIS_STREAM_MIN_NNZ, LAPIS_SPLIT_BLOCK_BYTES, LAPIS_SPLIT_MAX_BLOCKS,
 *  LAPIS_HUGE_ROW, LAPIS_LDS_BLOCK_BYTES}. */
int lapis_partition_constants(int64_t h_out[10]);

/* ---- host-side buffers with lazy synchronisation (after Section 4.3) ---------
 * A dual view pairs a pinned host buffer with a device buffer of the same size and keeps one
 * "modified" flag per side.  lapis_dualview_modify_host / _device only set a flag;
 * lapis_dualview_sync_device / _host copy the whole allocation to the named side only if the
 * other side was modified since the last sync, so a sync with nothing to do costs a flag test
 * (Section 4.3: lazy kokkos.sync / kokkos.modify instead of copying every buffer around every
 * kernel).  A sync while both sides are marked modified returns LAPIS_ERR_INVALID_ARG.
 * lapis_dualview_sync_host also synchronises the stream, so the host may read at once.
 * lapis_dualview_subview creates a view of `bytes` bytes at `offset_bytes` inside a parent: it
 * aliases the parent's memory, shares its flags (syncing a sub-view syncs the whole parent) and
 * keeps the memory alive until the last view of the allocation is destroyed.
 * lapis_dualview_host returns a HOST pointer, lapis_dualview_device a device pointer.
 * lapis_dualview_copy_counts reports how many host-to-device and device-to-host copies the
 * allocation has actually performed.
 * lapis_spmv_dualview: y = alpha*A*x + beta*y on dual views holding x (ncols values) and y
 * (nrows values) of A's dtype: syncs x and y to the device if needed (y's host copy is dropped
 * instead when beta == 0 and y is a whole allocation of exactly nrows values), runs
 * lapis_spmv, marks y modified on the device.  x and y may be sub-views of one allocation but must not overlap; a view smaller than
 * its operand is LAPIS_ERR_INVALID_ARG.  All functions here return a LAPIS_* status except the
 * two pointer getters (NULL for a NULL view); lapis_dualview_destroy(NULL) is a no-op.
 */
typedef struct lapis_dualview lapis_dualview_t;
int lapis_dualview_create(lapis_dualview_t **out, int64_t bytes);
int lapis_dualview_subview(lapis_dualview_t **out, lapis_dualview_t *parent, int64_t offset_bytes,
                           int64_t bytes);
void *lapis_dualview_host(lapis_dualview_t *v);
void *lapis_dualview_device(lapis_dualview_t *v);
int lapis_dualview_modify_host(lapis_dualview_t *v);
int lapis_dualview_modify_device(lapis_dualview_t *v);
int lapis_dualview_sync_device(lapis_dualview_t *v, void *hip_stream);
int lapis_dualview_sync_host(lapis_dualview_t *v, void *hip_stream);
int lapis_dualview_copy_counts(const lapis_dualview_t *v, int64_t *h2d, int64_t *d2h);
int lapis_dualview_destroy(lapis_dualview_t *v);
int lapis_spmv_dualview(const lapis_csr_t *A, double alpha, lapis_dualview_t *x, double beta,
                        lapis_dualview_t *y, void *hip_stream);

/*
 * lapis_batched_gemm - C[b] = alpha * A[b] * B[b] + beta * C[b] for b = 0 .. batch-1, many small
 * dense products (Section 5 of the paper: the batched kernel, for which the batch dimension is
 * the one to vectorise because the matrices themselves are small).
 *   d_A  DEVICE [batch][m][k], d_B  DEVICE [batch][k][n], d_C  DEVICE [batch][m][n], values of
 *        `dtype` (LAPIS_F32 / LAPIS_F64), every matrix row-major and the matrices of an operand
 *        back to back (a contiguous (batch, rows, cols) tensor); borrowed for the call; C must
 *        not overlap A or B
 *   1 <= m, n, k <= LAPIS_BATCHED_MAX_DIM; batch >= 0 (0: nothing is done, pointers may be NULL)
 *   alpha, beta are rounded to dtype; beta == 0: C is write-only (NaN or Inf in old C does not
 *   propagate)
 * Every element is one dot product of k terms accumulated in dtype with fused multiply-adds; the
 * order of the terms depends on the sizes only (small entries: l = 0 .. k-1; larger ones, on the
 * matrix cores: another fixed order), so equal calls give equal results.
 * Asynchronous on hip_stream (NULL = default stream): no allocation, no copy, no host
 * synchronisation.  Errors: LAPIS_ERR_INVALID_ARG (sizes out of range, NULL operand with
 * batch > 0), LAPIS_ERR_UNSUPPORTED (dtype), LAPIS_ERR_DEVICE (launch failure).
 */
#define LAPIS_BATCHED_MAX_DIM 32
int lapis_batched_gemm(int64_t batch, int32_t m, int32_t n, int32_t k, double alpha, const void *d_A,
                       const void *d_B, double beta, void *d_C, int dtype, void *hip_stream);

/* Text of the most recent error on the calling thread ("" if none).  The
 * pointer stays valid until the next failing call on that thread. */
const char *lapis_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* LAPIS_H */
