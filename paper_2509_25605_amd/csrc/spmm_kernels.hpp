// SpMM kernels for gfx950: Y = alpha*A*X + beta*Y, X and Y row-major; column c
// of Y is the SpMV of Section 6.2 applied to column c of X.
//
// A "slot" is CL consecutive lanes; lane l of a slot owns columns
// c0 + l*VEC .. c0 + l*VEC + VEC-1, so one slot reads one row of X with a single
// coalesced load (k = 16 doubles = one 128-byte line with CL = 8, VEC = 2).
//
//  * spmm_stream_kernel (rows of stream chunks): one wavefront per chunk of 32
//    rows.  The chunk's (column, value) pairs are streamed into LDS exactly as in
//    the SpMV stream kernel; then 64/CL slots walk 64/CL rows at a time, reading
//    each pair back as an LDS broadcast and one row of X with a 16-byte load per
//    lane, in whole batches of 16 / 8 / 4 / 2 / 1 entries while all rows of the
//    wavefront have that many left.  Consecutive rows sit in consecutive slots, so
//    on banded matrices one load instruction reads consecutive rows of X.
//  * spmm_rows_kernel (other rows of up to 64 entries): one slot per row.  The slot's
//    lanes load CL consecutive (column, value) pairs of the row at once, park
//    them in LDS, and every lane then reads them back one by one as LDS
//    broadcasts - each matrix entry is fetched from memory once and reused for
//    all k columns.
//  * spmm_block_rows_kernel (longer rows): one workgroup per row, slots stride
//    the row's entries, partial sums meet in LDS.
#pragma once
#include "device_utils.hpp"
#include "spmv_kernels.hpp"

namespace lapis {

template <typename T, int VEC>
struct alignas(sizeof(T) * VEC) Pack {
    T v[VEC];
};

template <typename T, int VEC>
__device__ __forceinline__ void store_row(T *__restrict__ yrow, const T (&acc)[VEC], int64_t col,
                                          int64_t k, T alpha, T beta)
{
    if (col >= k) return;
    if constexpr (VEC > 1) {
        Pack<T, VEC> out;
        if (beta == T(0)) {
#pragma unroll
            for (int q = 0; q < VEC; ++q) out.v[q] = alpha * acc[q];
        } else {
            const Pack<T, VEC> old = *reinterpret_cast<const Pack<T, VEC> *>(yrow + col);
#pragma unroll
            for (int q = 0; q < VEC; ++q) out.v[q] = alpha * acc[q] + beta * old.v[q];
        }
        *reinterpret_cast<Pack<T, VEC> *>(yrow + col) = out;
    } else {
        yrow[col] = (beta == T(0)) ? alpha * acc[0] : alpha * acc[0] + beta * yrow[col];
    }
}


// Columns [c0, min(c0 + CL*VEC, k)) of Y for the rows of the stream chunks.
// One wavefront (= one workgroup) per chunk; stream_chunks == nullptr means
// every chunk of the matrix.  colidx and vals 16-byte aligned, nnz4 = nnz & ~3.
// xcd_block == 0: each XCD owns a contiguous stretch of the chunk list; otherwise chunks are
// dealt to the XCDs block-cyclically, xcd_block chunks at a time (see xcd_block_cyclic_id).
constexpr int kSpmmUnroll = 16;  // X rows in flight per lane and batch

// ALL16: every listed chunk has 16-bit column offsets; the LDS window keeps them as 2-byte values.
//
// WINDOW (needs R >= 2 rows per slot and rows of X shorter than 64 KiB; pats = the row patterns
// of the matrix, ncols its columns): a chunk whose rows repeat the diagonals of its longest row,
// or ordered subsets of them, is worked on differently, from the values and the pattern table
// alone (no column index is read).  A slot takes R CONSECUTIVE rows (4 with 8 lanes per row of
// X, 8 with 16), and for every 3 consecutive diagonals d, d+1, d+2 of that longest row it loads
// the rows r0+d .. r0+d+R+1 of X once: row r0+p needs X rows r0+p+d+e = the p+e-th of them, so
// R + 2 loads serve 3 R products (a stencil's neighbouring rows share two thirds of their columns).  Rows with fewer diagonals
// (grid boundaries) carry a bit mask of the diagonals they have and skip the others.  Chunks
// that do not qualify take the ordinary path.
template <typename T, int VEC, int CL, bool XCD_REMAP, bool ALL16 = false, bool WINDOW = false>
__global__ __launch_bounds__(kWave) void spmm_stream_kernel(
    int32_t nrows, int32_t nnz, uint32_t num_chunks, uint32_t padded_chunks,
    const int32_t *__restrict__ stream_chunks, const int32_t *__restrict__ rowptr,
    uint32_t xcd_block, const int32_t *__restrict__ colidx, const int32_t *__restrict__ chunk_base,
    const int32_t *__restrict__ frame_table, const uint16_t *__restrict__ col16,
    const T *__restrict__ vals, int64_t k,
    int64_t c0, const T *__restrict__ X, int64_t ldx, T *__restrict__ Y, int64_t ldy, T alpha, T beta,
    StreamPatterns pats = StreamPatterns{nullptr, nullptr, nullptr}, int32_t ncols = 0)
{
    static_assert(CL <= 16, "column blocks wider than 16 lanes are split by the host");
    constexpr int kSlots = (kWave / CL > kStreamRows) ? kStreamRows : kWave / CL;
    constexpr int kPasses = kStreamRows / kSlots;
    __shared__ __attribute__((aligned(16))) T s_val[kStreamWindow];
    typedef typename std::conditional<ALL16, uint16_t, int32_t>::type idx_t;
    __shared__ __attribute__((aligned(16))) idx_t s_col[kStreamWindow];
    __shared__ int32_t s_rp[kStreamRows + 1];
    __shared__ int32_t s_tab[ALL16 ? 1 : kFrameSlots];

    const uint32_t id = !XCD_REMAP ? blockIdx.x
                        : xcd_block ? xcd_block_cyclic_id(blockIdx.x, xcd_block)
                                    : xcd_contiguous_id(blockIdx.x, padded_chunks);
    if (id >= num_chunks) return;
    const int lane = threadIdx.x;
    const int slot = lane / CL;
    const int l = lane % CL;
    const int64_t chunk = stream_chunks ? stream_chunks[id] : (int64_t)id;
    const int64_t row0 = chunk * kStreamRows;
    const int32_t cbase = chunk_base ? chunk_base[chunk] : -1;          // wave-uniform
    if constexpr (!ALL16) load_frame_table(frame_table, chunk, cbase, lane, s_tab);
    if (lane <= kStreamRows) {
        const int64_t r = row0 + lane;
        s_rp[lane] = rowptr[r < nrows ? r : nrows];     // rows past the end: empty
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const int32_t base = s_rp[0], end = s_rp[kStreamRows];
    const int32_t nnz4 = nnz & ~3;
    const int64_t col = c0 + (int64_t)l * VEC;
    const bool active = slot < kSlots && col < k;
    // Row c of X for this lane.  With 16-bit offsets (ALL16; the host guarantees a row of X is
    // shorter than 64 KiB) the row is a 32-bit byte offset from the chunk's base row: one 24-bit
    // multiply-add and a load with a scalar base; otherwise 64-bit pointer arithmetic.
    const uint32_t row_bytes = (uint32_t)(ldx * (int64_t)sizeof(T));
    auto x_row = [&](int32_t c) {
        if constexpr (ALL16)
            return *reinterpret_cast<const Pack<T, VEC> *>(
                reinterpret_cast<const char *>(X + (int64_t)cbase * ldx) +
                (__umul24((uint32_t)c, row_bytes) + (uint32_t)(col * (int64_t)sizeof(T))));
        else
            return *reinterpret_cast<const Pack<T, VEC> *>(X + (int64_t)c * ldx + col);
    };

    T acc[kPasses][VEC];
#pragma unroll
    for (int p = 0; p < kPasses; ++p)
#pragma unroll
        for (int q = 0; q < VEC; ++q) acc[p][q] = T(0);

    if constexpr (WINDOW) {
        static_assert(kPasses >= 2 && kSlots * kPasses == kStreamRows, "a slot takes kPasses consecutive rows");
        constexpr int R = kPasses;                 // consecutive rows of a slot: R + 2 rows of X serve 3 R products
        // the pattern table takes the place of the column window, which this path does not fill
        static_assert(kPatternTable * sizeof(int32_t) <= kStreamWindow * sizeof(idx_t), "the table fits the column window");
        int32_t *s_pat = reinterpret_cast<int32_t *>(s_col);
        __shared__ int32_t s_rowpat[kStreamRows];
        constexpr int kMaxOddRows = 4;            // more rows with a list of their own: the ordinary path
        constexpr int kOddBatch = 3;              // rows of X in flight per lane for such a row (kSlots times as many entries)
        const int32_t w0 = base & ~7;
        const int32_t pat_begin = pats.pat_off[chunk];
        const int32_t pat_len = pats.pat_off[chunk + 1] - pat_begin;   // wave-uniform; 0: not patterned
        if (pat_len > 0 && end - w0 <= kStreamWindow) {
            // the chunk's pattern table, and lane r < 32: row r of the chunk
            constexpr int kLoads = kPatternTable / kWave;
#pragma unroll
            for (int i = 0; i < kLoads; ++i)
                if (i * kWave < pat_len) s_pat[i * kWave + lane] = (i * kWave + lane < pat_len) ? pats.pool[pat_begin + i * kWave + lane] : 0;
            const int64_t my_row = row0 + (lane < kStreamRows ? lane : 0);
            const int32_t my_len = (lane < kStreamRows) ? s_rp[lane + 1] - s_rp[lane] : 0;
            const int32_t my_pat = (lane < kStreamRows && my_row < nrows && my_len > 0) ? (int32_t)pats.row_pat[my_row] : 0;
            // the values are needed either way and their loads overlap those above; no column is read here
            stream_values_to_lds<T>(vals, w0, end, nnz4, lane, s_val);     // ends with the wavefront's fence
            // the reference list: the diagonals of the first longest row, one per lane
            const int32_t ref_len = wave_max_nonneg(my_len);
            const uint64_t longest = __builtin_amdgcn_ballot_w64(my_len == ref_len);
            const int ref_lane = (int)__builtin_ctzll(longest);
            const int32_t ref_pat = __builtin_amdgcn_readlane(my_pat, ref_lane);
            // rows with another list (grid boundaries, empty rows, rows past the end): computed apart
            const bool is_row = lane < kStreamRows;
            const uint64_t odd = __builtin_amdgcn_ballot_w64(is_row && !(my_len == ref_len && my_pat == ref_pat));
            // the values of a row with the reference list are read at fixed places up to ref_len past
            // the start of ANY row, so that much room has to be left in the window
            bool all_ok = ref_len <= kWave && __popcll(odd) <= kMaxOddRows && end - w0 + kWave <= kStreamWindow;
            int32_t pstar = 0;
            if (all_ok) {
                const bool in_ref = lane < ref_len;
                pstar = in_ref ? s_pat[ref_pat + lane] : 0;
                const int32_t before = (in_ref && lane > 0) ? s_pat[ref_pat + lane - 1] : INT32_MIN;
                all_ok = __builtin_amdgcn_ballot_w64(in_ref && lane > 0 && pstar <= before) == 0;   // ascends strictly
                // the runs of consecutive diagonals have to come in whole threes (27-point stencils, blocks
                // of 3 unknowns): the loop below takes three diagonals and R + 2 rows of X at a time
                const uint64_t breaks = __builtin_amdgcn_ballot_w64(in_ref && (lane == 0 || pstar != before + 1));
                all_ok = all_ok && ref_len % 3 == 0 && (breaks & ~0x9249249249249249ull) == 0;
                // rows of X are addressed by 32-bit byte offsets from the row of the smallest diagonal
                const int64_t span = (int64_t)__builtin_amdgcn_readlane(pstar, ref_len - 1) - __builtin_amdgcn_readlane(pstar, 0) + 2 * kStreamRows;
                all_ok = all_ok && span < (1 << 24) && span * (int64_t)row_bytes < ((int64_t)1 << 31);
                if (is_row) s_rowpat[lane] = my_pat;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            if (all_ok) {
                if (active) {
                    const int r0 = slot * R;
                    int32_t first[R];
#pragma unroll
                    for (int pp = 0; pp < R; ++pp) first[pp] = s_rp[r0 + pp] - w0;
                    // X row (r0 + d + q) as an offset from the row of the smallest diagonal, kept inside X
                    // (a row of X that only an odd row's place would ask for may lie outside)
                    int64_t base_row = row0 + __builtin_amdgcn_readlane(pstar, 0);                 // uniform
                    base_row = base_row < 0 ? 0 : (base_row > ncols - 1 ? ncols - 1 : base_row);
                    const char *x_base = reinterpret_cast<const char *>(X + base_row * ldx);
                    const int32_t rel0 = (int32_t)(row0 + r0 - base_row);
                    const int32_t rel_max = (int32_t)(ncols - 1 - base_row);
                    auto x_at = [&](int32_t d, int q) {
                        int32_t rel = rel0 + d + q;
                        rel = rel < 0 ? 0 : (rel > rel_max ? rel_max : rel);
                        return *reinterpret_cast<const Pack<T, VEC> *>(
                            x_base + (__umul24((uint32_t)rel, row_bytes) + (uint32_t)(col * (int64_t)sizeof(T))));
                    };
                    constexpr int kRuns = R <= 4 ? 3 : 2;              // runs whose rows of X are in flight together
#pragma unroll 1
                    for (int t0 = 0; t0 < ref_len; t0 += 3 * kRuns) {  // uniform
                        Pack<T, VEC> xw[kRuns][R + 2];
#pragma unroll
                        for (int rr = 0; rr < kRuns; ++rr) {
                            if (t0 + 3 * rr < ref_len) {               // uniform
                                const int32_t d = __builtin_amdgcn_readlane(pstar, t0 + 3 * rr);
#pragma unroll
                                for (int q = 0; q < R + 2; ++q) xw[rr][q] = x_at(d, q);
                            }
                        }
#pragma unroll
                        for (int rr = 0; rr < kRuns; ++rr) {
                            const int tb = t0 + 3 * rr;
                            if (tb >= ref_len) continue;               // uniform
                            T v[3][R];
#pragma unroll
                            for (int e = 0; e < 3; ++e)
#pragma unroll
                                for (int pp = 0; pp < R; ++pp) v[e][pp] = s_val[first[pp] + tb + e];
#pragma unroll
                            for (int e = 0; e < 3; ++e)
#pragma unroll
                                for (int pp = 0; pp < R; ++pp)
#pragma unroll
                                    for (int q = 0; q < VEC; ++q)
                                        acc[pp][q] = fused_madd(v[e][pp], xw[rr][pp + e].v[q], acc[pp][q]);
                        }
                    }
                }
                // the odd rows: what the loop above left in their sums is discarded.  All slots share the
                // entries of such a row (slot s takes entries s, s + kSlots, ...), their partial sums are
                // added across the slots, and the slot that owns the row keeps the total
                {
                    const int r0 = slot * R;
                    for (uint64_t left = odd; left != 0; left &= left - 1) {               // uniform
                        const int row = (int)__builtin_ctzll(left);
                        const int n = s_rp[row + 1] - s_rp[row];                           // uniform
                        const int32_t *pat = s_pat + s_rowpat[row];
                        const T *sv = s_val + (s_rp[row] - w0);
                        const int64_t me = row0 + row;
                        T sum[VEC];
#pragma unroll
                        for (int q = 0; q < VEC; ++q) sum[q] = T(0);
                        for (int u0 = 0; u0 < n; u0 += kOddBatch * kSlots) {               // uniform
                            Pack<T, VEC> xo[kOddBatch];
                            T vo[kOddBatch];
#pragma unroll
                            for (int t = 0; t < kOddBatch; ++t) {
                                const int want = u0 + t * kSlots + slot;
                                const int u = want < n ? want : n - 1;                    // past the end: repeat
                                vo[t] = sv[u];
                                if (active) {
                                    xo[t] = *reinterpret_cast<const Pack<T, VEC> *>(X + (me + pat[u]) * ldx + col);
                                } else {
#pragma unroll
                                    for (int q = 0; q < VEC; ++q) xo[t].v[q] = T(0);
                                }
                            }
#pragma unroll
                            for (int t = 0; t < kOddBatch; ++t)
#pragma unroll
                                for (int q = 0; q < VEC; ++q)
                                    sum[q] += (active && u0 + t * kSlots + slot < n) ? vo[t] * xo[t].v[q] : T(0);
                        }
                        // lanes l, l + CL, l + 2 CL, ... hold the same columns: butterfly over the slots
#pragma unroll
                        for (int q = 0; q < VEC; ++q)
#pragma unroll
                            for (int step = CL; step < kWave; step *= 2) sum[q] += __shfl_xor(sum[q], step);
#pragma unroll
                        for (int pp = 0; pp < R; ++pp)
                            if (row == r0 + pp) {
#pragma unroll
                                for (int q = 0; q < VEC; ++q) acc[pp][q] = sum[q];
                            }
                    }
                }
                if (active) {
                    const int r0 = slot * R;
#pragma unroll
                    for (int pp = 0; pp < R; ++pp) {
                        const int64_t row = row0 + r0 + pp;
                        if (row < nrows) store_row<T, VEC>(Y + row * ldy, acc[pp], col, k, alpha, beta);
                    }
                }
                return;
            }
            // not all rows fit the reference list: the ordinary path
        }
    }
    for (int32_t w0 = base & ~7; w0 < end; w0 += kStreamWindow) {      // uniform
        const int32_t w1 = (end - w0 < kStreamWindow) ? end : w0 + kStreamWindow;
        stream_window_to_lds<T, idx_t>(colidx, col16, cbase, s_tab, vals, w0, w1, nnz4, lane, s_col, s_val);
#pragma unroll
        for (int p = 0; p < kPasses; ++p) {
            const int r = active ? p * kSlots + slot : 0;
            const int32_t rb = s_rp[r], re = s_rp[r + 1];
            const int32_t ub = (rb > w0 ? rb : w0) - w0;
            const int32_t ue = (re < w1 ? re : w1) - w0;
            const int n = active ? ue - ub : 0;                        // <= 0: row not in this window
            const int first = n > 0 ? ub : 0;
            const int last_u = n > 0 ? n - 1 : 0;
            const int n_all = wave_max_nonneg(n > 0 ? n : 0);          // every lane takes part
            if (active) {
                // While every lane in this branch still has B entries left (B = 16, then 8, 4, 2, 1),
                // a batch of B runs without clamps or selects: LDS reads at immediate offsets, one
                // address operation per row of X, fused multiply-adds.  What is left when the rows
                // of the wavefront differ in length goes through the ragged batches below, which
                // repeat a lane's last entry and discard the product.
                int u0 = 0;
                auto whole_batch = [&](auto batch) {
                    constexpr int B = decltype(batch)::value;
                    int32_t cj[B];
                    T vj[B];
                    Pack<T, VEC> xv[B];
                    const idx_t *sc = s_col + first + u0;
                    const T *sv = s_val + first + u0;
#pragma unroll
                    for (int t = 0; t < B; ++t) {
                        cj[t] = (int32_t)sc[t];
                        vj[t] = sv[t];
                    }
#pragma unroll
                    for (int t = 0; t < B; ++t) xv[t] = x_row(cj[t]);
#pragma unroll
                    for (int t = 0; t < B; ++t)
#pragma unroll
                        for (int q = 0; q < VEC; ++q) acc[p][q] = fused_madd(vj[t], xv[t].v[q], acc[p][q]);
                    u0 += B;
                };
                auto all_have = [&](int b) { return __builtin_amdgcn_ballot_w64(n - u0 < b) == 0; };
#pragma unroll 1
                while (all_have(kSpmmUnroll)) whole_batch(std::integral_constant<int, kSpmmUnroll>());
                if (all_have(8)) whole_batch(std::integral_constant<int, 8>());
                if (all_have(4)) whole_batch(std::integral_constant<int, 4>());
                if (all_have(2)) whole_batch(std::integral_constant<int, 2>());
                if (all_have(1)) whole_batch(std::integral_constant<int, 1>());
#pragma unroll 1
                for (; u0 < n_all; u0 += kSpmmUnroll) {
                    if (u0 >= n) continue;
                    int32_t cj[kSpmmUnroll];
                    T vj[kSpmmUnroll];
                    Pack<T, VEC> xv[kSpmmUnroll];
#pragma unroll
                    for (int t = 0; t < kSpmmUnroll; ++t) {
                        const int u = first + (u0 + t < last_u ? u0 + t : last_u);  // past the end: repeat
                        cj[t] = (int32_t)s_col[u];
                        vj[t] = s_val[u];
                    }
#pragma unroll
                    for (int t = 0; t < kSpmmUnroll; ++t) xv[t] = x_row(cj[t]);
#pragma unroll
                    for (int t = 0; t < kSpmmUnroll; ++t)
#pragma unroll
                        for (int q = 0; q < VEC; ++q) acc[p][q] += (u0 + t < n) ? vj[t] * xv[t].v[q] : T(0);
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    if (active) {
#pragma unroll
        for (int p = 0; p < kPasses; ++p) {
            const int64_t row = row0 + p * kSlots + slot;
            if (row < nrows) store_row<T, VEC>(Y + row * ldy, acc[p], col, k, alpha, beta);
        }
    }
}

// positions [0, count) of row_perm, one slot per row.
template <typename T, int VEC, int CL, bool XCD_REMAP>
__global__ __launch_bounds__(kBlock) void spmm_rows_kernel(
    int32_t count, uint32_t num_blocks, uint32_t padded_blocks,
    const int32_t *__restrict__ row_perm, const int32_t *__restrict__ rowptr,
    const int32_t *__restrict__ colidx, const T *__restrict__ vals, int64_t k,
    const T *__restrict__ X, int64_t ldx, T *__restrict__ Y, int64_t ldy, T alpha, T beta)
{
    constexpr int kSlots = kBlock / CL;
    __shared__ int32_t s_col[kBlock];
    __shared__ T s_val[kBlock];

    const uint32_t id = XCD_REMAP ? xcd_contiguous_id(blockIdx.x, padded_blocks) : blockIdx.x;
    if (id >= num_blocks) return;
    const int slot = threadIdx.x / CL;
    const int l = threadIdx.x % CL;
    const int64_t idx = (int64_t)id * kSlots + slot;
    if (idx >= count) return;  // whole slots leave together; the rest of the wave carries on
    const int32_t row = row_perm[idx];
    const int64_t jb = rowptr[row], je = rowptr[row + 1];
    T *__restrict__ yrow = Y + (int64_t)row * ldy;

    for (int64_t c0 = 0; c0 < k; c0 += CL * VEC) {
        const int64_t col = c0 + (int64_t)l * VEC;
        const bool col_ok = col < k;
        T acc[VEC];
#pragma unroll
        for (int q = 0; q < VEC; ++q) acc[q] = T(0);
        for (int64_t j0 = jb; j0 < je; j0 += CL) {
            // all lanes of the slot take part in the exchange; LDS operations of
            // one wavefront execute in program order
            const int64_t j = j0 + l;
            s_col[threadIdx.x] = (j < je) ? load_stream(colidx + j) : 0;
            s_val[threadIdx.x] = (j < je) ? load_stream(vals + j) : T(0);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const int n_here = (je - j0 < CL) ? (int)(je - j0) : CL;
            if (col_ok) {
                // Entries past the end of the row re-read the last valid one (same
                // X line, no new traffic) and their product is discarded, so all CL
                // loads can be issued back to back without branches.
#pragma unroll
                for (int t = 0; t < CL; ++t) {
                    const int tt = (t < n_here) ? t : n_here - 1;
                    const int32_t cj = s_col[slot * CL + tt];
                    const T vj = s_val[slot * CL + tt];
                    const T *__restrict__ xr = X + (int64_t)cj * ldx + col;
                    if constexpr (VEC > 1) {
                        const Pack<T, VEC> xv = *reinterpret_cast<const Pack<T, VEC> *>(xr);
#pragma unroll
                        for (int q = 0; q < VEC; ++q) acc[q] += (t < n_here) ? vj * xv.v[q] : T(0);
                    } else {
                        acc[0] += (t < n_here) ? vj * xr[0] : T(0);
                    }
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
        store_row<T, VEC>(yrow, acc, col, k, alpha, beta);
    }
}

// positions [first, first+count) of row_perm, one workgroup per row.
template <typename T, int VEC, int CL>
__global__ __launch_bounds__(kBlock) void spmm_block_rows_kernel(
    int32_t first, const int32_t *__restrict__ row_perm, const int32_t *__restrict__ rowptr,
    const int32_t *__restrict__ colidx, const T *__restrict__ vals, int64_t k,
    const T *__restrict__ X, int64_t ldx, T *__restrict__ Y, int64_t ldy, T alpha, T beta)
{
    constexpr int kSlots = kBlock / CL;
    __shared__ T red[kBlock * VEC];  // [slot][lane*VEC + q]

    const int slot = threadIdx.x / CL;
    const int l = threadIdx.x % CL;
    const int32_t row = row_perm[first + (int64_t)blockIdx.x];
    const int64_t jb = rowptr[row], je = rowptr[row + 1];
    T *__restrict__ yrow = Y + (int64_t)row * ldy;

    for (int64_t c0 = 0; c0 < k; c0 += CL * VEC) {
        const int64_t col = c0 + (int64_t)l * VEC;
        T acc[VEC];
#pragma unroll
        for (int q = 0; q < VEC; ++q) acc[q] = T(0);
        if (col < k) {
            for (int64_t j = jb + slot; j < je; j += kSlots) {
                const int32_t cj = load_stream(colidx + j);
                const T vj = load_stream(vals + j);
                const T *__restrict__ xr = X + (int64_t)cj * ldx + col;
                if constexpr (VEC > 1) {
                    const Pack<T, VEC> xv = *reinterpret_cast<const Pack<T, VEC> *>(xr);
#pragma unroll
                    for (int q = 0; q < VEC; ++q) acc[q] += vj * xv.v[q];
                } else {
                    acc[0] += vj * xr[0];
                }
            }
        }
#pragma unroll
        for (int q = 0; q < VEC; ++q) red[(slot * CL + l) * VEC + q] = acc[q];
        __syncthreads();
        if (slot == 0) {
            T tot[VEC];
#pragma unroll
            for (int q = 0; q < VEC; ++q) tot[q] = T(0);
            for (int s = 0; s < kSlots; ++s) {
#pragma unroll
                for (int q = 0; q < VEC; ++q) tot[q] += red[(s * CL + l) * VEC + q];
            }
            store_row<T, VEC>(yrow, tot, col, k, alpha, beta);
        }
        __syncthreads();
    }
}

}  // namespace lapis
