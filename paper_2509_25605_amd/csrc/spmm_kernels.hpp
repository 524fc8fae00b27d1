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
//    Launches over few chunks of long rows give every pass of a chunk (the rows
//    the slots take together) a wavefront of its own.
//  * spmm_shared_kernel (stream chunks whose rows repeat one list of diagonals):
//    a slot takes 4 or 8 consecutive rows and loads the rows of X that they have
//    in common once; no column index is read.  spmm_block_shared_kernel does the
//    same for the rows of grid points with 2 or 3 unknowns.  Which chunks these
//    are is decided once per matrix (spmm_share_flag_kernel).
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

// One lane's VEC columns of a row of Y.  Non-temporal stores: Y is written once per product and, at
// k = 16 doubles, is 16 times as large as a vector, so it leaves the L2 to the rows of X that come
// back (workload 5: 254 -> 245 us, 7-point and 5-point grids 3 to 5 %).
template <typename T, int VEC>
__device__ __forceinline__ void store_row(T *__restrict__ yrow, const T (&acc)[VEC], int64_t col,
                                          int64_t k, T alpha, T beta)
{
    if (col >= k) return;
    if constexpr (VEC > 1) {
        typedef T vec_t __attribute__((ext_vector_type(VEC)));
        vec_t out;
        if (beta == T(0)) {
#pragma unroll
            for (int q = 0; q < VEC; ++q) out[q] = alpha * acc[q];
        } else {
            const Pack<T, VEC> old = *reinterpret_cast<const Pack<T, VEC> *>(yrow + col);
#pragma unroll
            for (int q = 0; q < VEC; ++q) out[q] = alpha * acc[q] + beta * old.v[q];
        }
        __builtin_nontemporal_store(out, reinterpret_cast<vec_t *>(yrow + col));
    } else {
        const T out = (beta == T(0)) ? alpha * acc[0] : alpha * acc[0] + beta * yrow[col];
        __builtin_nontemporal_store(out, yrow + col);
    }
}


// Columns [c0, min(c0 + CL*VEC, k)) of Y for the rows of the stream chunks.
// One wavefront (= one workgroup) per chunk; stream_chunks == nullptr means
// every chunk of the matrix.  colidx and vals 16-byte aligned, nnz4 = nnz & ~3.
// xcd_block == 0: each XCD owns a contiguous stretch of the chunk list; otherwise chunks are
// dealt to the XCDs block-cyclically, xcd_block chunks at a time (see xcd_block_cyclic_id).
constexpr int kSpmmUnroll = 16;  // X rows in flight per lane and batch

// ALL16: every listed chunk has 16-bit column offsets; the LDS window keeps them as 2-byte values.
// PER_PASS: a chunk is shared by kPasses wavefronts, each taking the kSlots consecutive rows of one pass
// (num_chunks and padded_chunks then count those wavefronts): for launches over so few chunks that one
// wavefront per chunk would leave most of the GPU idle while each walks its 32 rows.
template <typename T, int VEC, int CL, bool XCD_REMAP, bool ALL16 = false, bool PER_PASS = false>
__global__ __launch_bounds__(kWave) void spmm_stream_kernel(
    int32_t nrows, int32_t nnz, uint32_t num_chunks, uint32_t padded_chunks,
    const int32_t *__restrict__ stream_chunks, const int32_t *__restrict__ rowptr,
    uint32_t xcd_block, const int32_t *__restrict__ colidx, const int32_t *__restrict__ chunk_base,
    const int32_t *__restrict__ frame_table, const uint16_t *__restrict__ col16,
    const T *__restrict__ vals, int64_t k,
    int64_t c0, const T *__restrict__ X, int64_t ldx, T *__restrict__ Y, int64_t ldy, T alpha, T beta)
{
    static_assert(CL <= 16, "column blocks wider than 16 lanes are split by the host");
    constexpr int kSlots = (kWave / CL > kStreamRows) ? kStreamRows : kWave / CL;
    constexpr int kParts = PER_PASS ? kStreamRows / kSlots : 1;      // wavefronts per chunk
    constexpr int kPasses = kStreamRows / kSlots / kParts;           // passes of one wavefront
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
    const uint32_t listed = id / kParts;
    const int first_row = (int)(id % kParts) * kPasses * kSlots;        // this wavefront's rows of the chunk
    const int64_t chunk = stream_chunks ? stream_chunks[listed] : (int64_t)listed;
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
    const int32_t base = s_rp[first_row], end = s_rp[first_row + kPasses * kSlots];
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

    for (int32_t w0 = base & ~7; w0 < end; w0 += kStreamWindow) {      // uniform
        const int32_t w1 = (end - w0 < kStreamWindow) ? end : w0 + kStreamWindow;
        stream_window_to_lds<T, idx_t>(colidx, col16, cbase, s_tab, vals, w0, w1, nnz4, lane, s_col, s_val);
#pragma unroll
        for (int p = 0; p < kPasses; ++p) {
            const int r = active ? first_row + p * kSlots + slot : 0;
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
            const int64_t row = row0 + first_row + p * kSlots + slot;
            if (row < nrows) store_row<T, VEC>(Y + row * ldy, acc[p], col, k, alpha, beta);
        }
    }
}

// ---- rows of X shared between neighbouring matrix rows ---------------------------------------
// On matrices of regular grids row i + 1 needs the rows of X that row i needs, shifted by one.  A
// chunk of 32 rows "shares rows" when (a) it is patterned (its rows repeat a few lists of diagonals
// = column - row, spmv_kernels.hpp), (b) its longest row's list - the reference list, at most 64
// diagonals - ascends strictly, (c) at most kShareMaxOdd of its rows are not "regular" (regular: the
// reference row's length, stored list and shift; the others, rows of grid boundaries or empty rows,
// are the "odd" rows), (d) its values fit one LDS window with 64 entries to spare
// (a row with the reference list reads its values at fixed places past the start of ANY row).
// The reference list is cut into runs of consecutive
// diagonals and every run into pieces of 3 and a rest of 2 or 1.  A slot (CL lanes = one row of
// X per load) takes R CONSECUTIVE rows r0 .. r0 + R - 1 (R = 4 with 8 lanes per row of X, 8 with
// 16); for a piece of LEN diagonals starting at d it loads the rows r0 + d .. r0 + d + R + LEN - 2
// of X once: row r0 + p multiplies its entry of diagonal d + e with the (p + e)-th of them, so
// R + LEN - 1 loads serve R * LEN products (6 for 12, 10 for 24).  No column index is read: the
// chunk is worked on from its values and its pattern table alone.
constexpr int kShareMaxOdd = 4;

// What a wavefront knows about its chunk after the first round trip; lane r < 32 holds row r.
// A row is regular when it has the reference row's length and stored list and, if `same_shift`, also its
// shift (the rows of a regular grid); without `same_shift` any shift will do (block rows, see
// spmm_share_flag_kernel).
struct ShareRows {
    int32_t my_rp, my_len, my_pat;     // lane r: first entry, length and packed pattern (start | shift << 9) of row r (0 past the end)
    int32_t base, end, w0;             // the chunk's entries [base, end), w0 = base rounded down to 8
    int32_t ref_len, ref_pat;          // the reference list: length, packed pattern of the row it is taken from
    uint64_t odd;                      // rows (below nrows) that are not regular
    bool few_odd;                      // (a), (c) and a reference list that is not empty
    bool one_window;                   // (d)
};

__device__ __forceinline__ ShareRows share_rows_setup(int lane, int32_t nrows, int64_t row0,
                                                      const int32_t *__restrict__ rowptr,
                                                      const uint16_t *__restrict__ row_pat, int32_t pat_len,
                                                      bool same_shift)
{
    ShareRows c;
    const bool is_row = lane < kStreamRows;
    const int64_t my_row = row0 + (is_row ? lane : kStreamRows);
    const int64_t my_row_c = my_row < nrows ? my_row : nrows;
    c.my_rp = rowptr[my_row_c];
    const int32_t my_re = rowptr[my_row_c < nrows ? my_row_c + 1 : nrows];
    c.my_len = is_row ? my_re - c.my_rp : 0;
    const int32_t pat_raw = (is_row && my_row < nrows) ? (int32_t)row_pat[my_row] : 0;
    c.my_pat = c.my_len > 0 ? pat_raw : 0;
    c.base = __builtin_amdgcn_readfirstlane(c.my_rp);
    c.end = __builtin_amdgcn_readlane(c.my_rp, kStreamRows);
    c.w0 = c.base & ~7;
    c.ref_len = wave_max_nonneg(c.my_len);
    const uint64_t longest = __builtin_amdgcn_ballot_w64(is_row && c.my_len == c.ref_len);
    c.ref_pat = __builtin_amdgcn_readlane(c.my_pat, (int)__builtin_ctzll(longest));
    const bool regular = c.my_len == c.ref_len &&
                         (same_shift ? c.my_pat == c.ref_pat : pattern_start(c.my_pat) == pattern_start(c.ref_pat));
    c.odd = __builtin_amdgcn_ballot_w64(is_row && my_row < nrows && !regular);
    c.few_odd = pat_len > 0 && c.ref_len > 0 && __popcll(c.odd) <= kShareMaxOdd;
    c.one_window = c.end - c.w0 + kWave <= kStreamWindow;
    return c;
}

// Minimum over the aligned groups of four lanes (quad permutes: lane ^ 1, lane ^ 2).
__device__ __forceinline__ int32_t quad_min(int32_t v)
{
    v = min(v, __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xf, 0xf, false));
    return min(v, __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xf, 0xf, false));
}

// Lane t holds diagonal t of a list of `count` diagonals (count <= 0: none, > 64: the first 64 of them).
// Every run of consecutive diagonals is cut into pieces of 3 and a rest of 2 or 1; a run also ends
// wherever t is a multiple of SEG.  Bit t of m3 / m2 / m1: a piece of that length starts at diagonal t.
template <int SEG>
__device__ __forceinline__ void share_piece_masks(int32_t pstar, int32_t count, int lane, uint64_t &m3,
                                                  uint64_t &m2, uint64_t &m1)
{
    const bool in_ref = lane < count;
    const int32_t before = __builtin_amdgcn_update_dpp(0, pstar, 0x138, 0xf, 0xf, false);   // lane t gets lane t - 1
    const uint64_t brk = __builtin_amdgcn_ballot_w64(in_ref && (lane % SEG == 0 || pstar != before + 1));   // run starts
    const uint64_t upto = (2ull << lane) - 1;                                  // lanes 0 .. this one
    const int run_start = 63 - (int)__builtin_clzll((brk & upto) | 1);
    const uint64_t past = (count > 0 && count < kWave) ? (1ull << count) : 0;
    const uint64_t above = (brk | past) & ~upto;
    const int run_end = above ? (int)__builtin_ctzll(above) : kWave;           // first lane past this lane's run
    const bool piece_start = in_ref && (lane - run_start) % 3 == 0;
    const int piece_len = run_end - lane < 3 ? run_end - lane : 3;
    m3 = __builtin_amdgcn_ballot_w64(piece_start && piece_len == 3);
    m2 = __builtin_amdgcn_ballot_w64(piece_start && piece_len == 2);
    m1 = __builtin_amdgcn_ballot_w64(piece_start && piece_len == 1);
}

// Analysis, one wavefront per chunk: flag_out[c] = 0 if c is not a stream chunk (stream_flag[c] == 0),
// kSharePlain if it shares rows of X as defined above, kShareBlock3 / kShareBlock2 if it does so with
// block rows (below), kShareNone otherwise.
// Block rows: the regular rows have the reference row's stored list with shifts of their own (the rows of
// the unknowns of one grid point hold the same columns), (a) to (c) hold with a reference list of at most
// kShareBlockMaxLen diagonals, and with v = (row + its shift) the regular rows of every aligned group of
// four (the rows of one slot of 8 lanes per row of X) have v equal to the group's smallest v or to that
// plus DELTA, with one DELTA (3 or 2) for the whole chunk and at least one row at DELTA: a group of four
// rows touches two grid points.
constexpr int32_t kSharePlain = 1, kShareNone = 2, kShareBlock3 = 3, kShareBlock2 = 4;
constexpr int kShareBlockMaxLen = 2 * kWave;
constexpr int kShareBlockSeg = 32;   // diagonals per pass of spmm_block_shared_kernel (64 is no faster and takes twice the LDS)
__global__ __launch_bounds__(kBlock) void spmm_share_flag_kernel(
    int32_t nrows, int32_t num_chunks, const int32_t *__restrict__ stream_flag,
    const int32_t *__restrict__ rowptr, StreamPatterns pats, int32_t *__restrict__ flag_out)
{
    const int64_t chunk = (int64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
    if (chunk >= num_chunks) return;                                       // whole wavefronts leave
    const int lane = threadIdx.x % kWave;
    int32_t result = 0;
    if (stream_flag[chunk] != 0) {
        result = kShareNone;
        const int64_t row0 = chunk * kStreamRows;
        const int32_t pat_begin = pats.pat_off[chunk];
        const int32_t pat_len = pats.pat_off[chunk + 1] - pat_begin;
        const ShareRows plain = share_rows_setup(lane, nrows, row0, rowptr, pats.row_pat, pat_len, true);
        const ShareRows block = share_rows_setup(lane, nrows, row0, rowptr, pats.row_pat, pat_len, false);
        if (block.few_odd && block.ref_len <= kShareBlockMaxLen) {         // uniform; plain.few_odd implies block.few_odd
            // the stored list must ascend strictly (a shift moves all diagonals alike)
            const int32_t *list = pats.pool + pat_begin + pattern_start(block.ref_pat);
            const int32_t d_lo = lane < block.ref_len ? list[lane] : 0;
            const int32_t d_hi = lane + kWave < block.ref_len ? list[lane + kWave] : 0;
            const int32_t before_lo = __builtin_amdgcn_update_dpp(0, d_lo, 0x138, 0xf, 0xf, false);   // lane t gets lane t - 1
            int32_t before_hi = __builtin_amdgcn_update_dpp(0, d_hi, 0x138, 0xf, 0xf, false);
            const int32_t last_lo = __builtin_amdgcn_readlane(d_lo, kWave - 1);
            if (lane == 0) before_hi = last_lo;
            const uint64_t descending = __builtin_amdgcn_ballot_w64(
                (lane > 0 && lane < block.ref_len && d_lo <= before_lo) || (lane + kWave < block.ref_len && d_hi <= before_hi));
            if (descending == 0) {
                if (plain.few_odd && plain.one_window && plain.ref_len <= kWave) result = kSharePlain;
                else {
                    const bool regular = lane < kStreamRows && row0 + lane < nrows && !((block.odd >> lane) & 1);
                    const int32_t v = lane + pattern_shift(block.my_pat);
                    const int32_t group_min = quad_min(regular ? v : INT32_MAX);      // every lane takes part
                    const int32_t diff = regular ? v - group_min : 0;
                    const uint64_t two = __builtin_amdgcn_ballot_w64(diff == 2), three = __builtin_amdgcn_ballot_w64(diff == 3);
                    const uint64_t other = __builtin_amdgcn_ballot_w64(diff != 0 && diff != 2 && diff != 3);
                    if (other == 0 && three != 0 && two == 0) result = kShareBlock3;
                    if (other == 0 && two != 0 && three == 0) result = kShareBlock2;
                }
            }
        }
    }
    if (lane == 0) flag_out[chunk] = result;
}

// An odd row (entries [rb, rb + n), packed pattern `packed`, values at `sv`, in LDS or in memory) of a
// chunk that shares rows of X, computed by all slots together: slot s takes the entries s, s + kSlots,
// ...; the partial sums meet in a butterfly of lane exchanges and the slot `owner` stores the row.  No
// product of an absent entry is formed.
template <typename T, int VEC, int CL>
__device__ __forceinline__ void share_odd_row(const T *sv, int32_t n, const int32_t *__restrict__ pat, int64_t me,
                                              int64_t me_x, int slot, bool owner, bool active, int64_t col, int64_t k,
                                              const T *__restrict__ X, int64_t ldx, T *__restrict__ Y, int64_t ldy,
                                              T alpha, T beta)
{
    constexpr int kSlots = kWave / CL;
    constexpr int kOddBatch = 3;                       // rows of X in flight per lane
    T sum[VEC];
#pragma unroll
    for (int q = 0; q < VEC; ++q) sum[q] = T(0);
    for (int u0 = 0; u0 < n; u0 += kOddBatch * kSlots) {                   // uniform
        Pack<T, VEC> xo[kOddBatch];
        T vo[kOddBatch];
        int32_t dd[kOddBatch];
#pragma unroll
        for (int t = 0; t < kOddBatch; ++t) {
            const int want = u0 + t * kSlots + slot;
            const int u = want < n ? want : n - 1;                        // past the end: repeat
            dd[t] = pat[u];
            vo[t] = sv[u];
        }
#pragma unroll
        for (int t = 0; t < kOddBatch; ++t) {
            if (active) xo[t] = *reinterpret_cast<const Pack<T, VEC> *>(X + (me_x + dd[t]) * ldx + col);
            else {
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
    if (active && owner) store_row<T, VEC>(Y + me * ldy, sum, col, k, alpha, beta);
}

// Columns [c0, min(c0 + CL*VEC, k)) of Y for chunks of share class kSharePlain: the listed chunks, or
// (stream_chunks == nullptr) every chunk of the matrix, of which those with another share_flag are
// skipped when share_flag is given.  One wavefront per chunk.  vals 16-byte aligned; a row of X shorter
// than 16 MiB (32-bit offsets of a lane from the wave-uniform row address).  The odd rows are computed
// first (share_odd_row), so a non-finite row of X reaches exactly the rows that hold its column.  What
// the main loop leaves in the sums of odd rows is never stored.  The pieces are taken longest first
// (all pieces of 3, then of 2, then of 1), NB of them in flight; a piece's registers are refilled as
// soon as it has been multiplied out.
template <typename T, int VEC, int CL, bool XCD_REMAP>
__global__ __launch_bounds__(kWave) __attribute__((amdgpu_waves_per_eu(CL <= 8 ? 4 : 2)))
void spmm_shared_kernel(
    int32_t nrows, int32_t nnz, uint32_t num_chunks, uint32_t padded_chunks,
    const int32_t *__restrict__ stream_chunks, const int32_t *__restrict__ share_flag,
    const int32_t *__restrict__ rowptr, uint32_t xcd_block,
    const T *__restrict__ vals, int64_t k, int64_t c0, const T *__restrict__ X, int64_t ldx, T *__restrict__ Y,
    int64_t ldy, T alpha, T beta, StreamPatterns pats, int32_t ncols)
{
    static_assert(CL == 8 || CL == 16, "a slot is 8 or 16 lanes");
    constexpr int kSlots = kWave / CL;
    constexpr int R = kStreamRows / kSlots;            // consecutive rows of a slot
    __shared__ __attribute__((aligned(16))) T s_val[kStreamWindow];

    const uint32_t id = !XCD_REMAP ? blockIdx.x
                        : xcd_block ? xcd_block_cyclic_id(blockIdx.x, xcd_block)
                                    : xcd_contiguous_id(blockIdx.x, padded_chunks);
    if (id >= num_chunks) return;
    const int lane = threadIdx.x;
    const int slot = lane / CL;
    const int l = lane % CL;
    const int64_t chunk = stream_chunks ? stream_chunks[id] : (int64_t)id;
    const int64_t row0 = chunk * kStreamRows;
    // round trip 1: row pointers, the rows' pattern starts, the chunk's place in the pool
    const int32_t flag = share_flag ? share_flag[chunk] : kSharePlain;     // wave-uniform
    const int32_t pat_begin = pats.pat_off[chunk];
    const ShareRows c = share_rows_setup(lane, nrows, row0, rowptr, pats.row_pat, 1, true);
    if (flag != kSharePlain) return;                                       // another kernel's chunk
    const int32_t w0 = c.w0;
    const int64_t col = c0 + (int64_t)l * VEC;
    const bool active = col < k;
    const uint32_t row_bytes = (uint32_t)(ldx * (int64_t)sizeof(T));
    // round trip 2: the values into LDS, the reference list one diagonal per lane
    const bool in_ref = lane < c.ref_len;
    const int32_t pstar = in_ref ? pats.pool[pat_begin + pattern_start(c.ref_pat) + lane] + pattern_shift(c.ref_pat) : 0;
    stream_values_to_lds<T>(vals, w0, c.end, nnz & ~3, lane, s_val);           // ends with the wavefront's fence
    uint64_t m3, m2, m1;                                                       // lane t: a piece starts at diagonal t
    share_piece_masks<kWave>(pstar, c.ref_len, lane, m3, m2, m1);

    const int r0 = slot * R;
    int32_t first[R];
#pragma unroll
    for (int pp = 0; pp < R; ++pp) first[pp] = __shfl(c.my_rp, r0 + pp) - w0;
    // row (row0 + r0 + d + q) of X = a wave-uniform address (row row0 + d + q) + this lane's fixed offset.
    // Every row of X that a slot of regular rows asks for is the column of one of its entries; a slot with
    // an odd row (or rows past the end) also asks for rows that no entry names.  Only near the ends of
    // the matrix can those lie outside X: such chunks (`inside` false) clamp every row number.
    const uint32_t lane_off = (uint32_t)r0 * row_bytes + (uint32_t)(col * (int64_t)sizeof(T));
    const char *x0 = reinterpret_cast<const char *>(X) + row0 * (int64_t)row_bytes;
    const int64_t d_min = __builtin_amdgcn_readlane(pstar, 0), d_max = __builtin_amdgcn_readlane(pstar, c.ref_len - 1);
    const bool inside = row0 + d_min >= 0 && row0 + kStreamRows + 1 + d_max <= (int64_t)ncols - 1;   // uniform

    for (uint64_t left = c.odd; left != 0; left &= left - 1) {               // uniform
        const int row = (int)__builtin_ctzll(left);
        const int32_t rb = __builtin_amdgcn_readlane(c.my_rp, row), n = __builtin_amdgcn_readlane(c.my_len, row);
        const int32_t packed = __builtin_amdgcn_readlane(c.my_pat, row);
        share_odd_row<T, VEC, CL>(s_val + (rb - w0), n, pats.pool + pat_begin + pattern_start(packed), row0 + row,
                                  row0 + row + pattern_shift(packed), slot, row / R == slot, active, col, k, X, ldx,
                                  Y, ldy, alpha, beta);
    }

    if (!active) return;
    T acc[R][VEC];
#pragma unroll
    for (int pp = 0; pp < R; ++pp)
#pragma unroll
        for (int q = 0; q < VEC; ++q) acc[pp][q] = T(0);
    auto run_class = [&](auto len_tag, auto inside_tag, uint64_t mask) {
        constexpr int LEN = decltype(len_tag)::value;
        constexpr bool kInside = decltype(inside_tag)::value;
        constexpr int NX = R + LEN - 1;                    // rows of X per piece
        constexpr int NB = !kInside ? 2 : R > 4 ? 2 : (LEN == 1 ? 4 : 3);   // pieces in flight (the rare clamped variant: fewer registers)
        Pack<T, VEC> xw[NB][NX];
        int tt[NB];
        auto fill = [&](int b) {
            tt[b] = (int)__builtin_ctzll(mask);
            mask &= mask - 1;
            const int32_t d = __builtin_amdgcn_readlane(pstar, tt[b]);
            const char *xb = x0 + (int64_t)d * (int64_t)row_bytes;            // uniform: scalar arithmetic
#pragma unroll
            for (int q = 0; q < NX; ++q) {
                if constexpr (kInside) {
                    xw[b][q] = *reinterpret_cast<const Pack<T, VEC> *>(xb + lane_off);
                    xb += row_bytes;
                } else {
                    int64_t r = row0 + r0 + d + q;
                    r = r < 0 ? 0 : (r > (int64_t)ncols - 1 ? (int64_t)ncols - 1 : r);
                    xw[b][q] = *reinterpret_cast<const Pack<T, VEC> *>(X + r * ldx + col);
                }
            }
        };
        auto use = [&](int b) {
            T v[LEN][R];
#pragma unroll
            for (int e = 0; e < LEN; ++e)
#pragma unroll
                for (int pp = 0; pp < R; ++pp) v[e][pp] = s_val[first[pp] + tt[b] + e];
#pragma unroll
            for (int e = 0; e < LEN; ++e)
#pragma unroll
                for (int pp = 0; pp < R; ++pp)
#pragma unroll
                    for (int q = 0; q < VEC; ++q) acc[pp][q] = fused_madd(v[e][pp], xw[b][pp + e].v[q], acc[pp][q]);
        };
        int left = __popcll(mask);                         // pieces not yet asked for
        if (left >= NB) {
#pragma unroll
            for (int b = 0; b < NB; ++b) fill(b);
            left -= NB;
#pragma unroll 1
            while (left >= NB) {                           // steady state: every piece multiplied out is replaced
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    use(b);
                    __builtin_amdgcn_sched_barrier(0);     // the refill stays below the products it replaces
                    fill(b);
                    __builtin_amdgcn_sched_barrier(0);
                }
                left -= NB;
            }
#pragma unroll
            for (int b = 0; b < NB; ++b) use(b);
            __builtin_amdgcn_sched_barrier(0);
        }
        // fewer than NB pieces are left
#pragma unroll
        for (int b = 0; b < NB - 1; ++b)
            if (b < left) fill(b);
#pragma unroll
        for (int b = 0; b < NB - 1; ++b)
            if (b < left) use(b);
    };
    if (inside) {
        if (m3) run_class(std::integral_constant<int, 3>(), std::true_type(), m3);
        if (m2) run_class(std::integral_constant<int, 2>(), std::true_type(), m2);
        if (m1) run_class(std::integral_constant<int, 1>(), std::true_type(), m1);
    } else {
        if (m3) run_class(std::integral_constant<int, 3>(), std::false_type(), m3);
        if (m2) run_class(std::integral_constant<int, 2>(), std::false_type(), m2);
        if (m1) run_class(std::integral_constant<int, 1>(), std::false_type(), m1);
    }
#pragma unroll
    for (int pp = 0; pp < R; ++pp) {
        const int64_t row = row0 + r0 + pp;
        if (row < nrows && !((c.odd >> (r0 + pp)) & 1)) store_row<T, VEC>(Y + row * ldy, acc[pp], col, k, alpha, beta);
    }
}

// Columns [c0, min(c0 + 8 VEC, k)) of Y for chunks of share class kShareBlock3 (DELTA 3) or kShareBlock2
// (DELTA 2), listed or by flag as above, `want_flag` being the class.  One wavefront per chunk, 8 lanes per
// row of X, a slot takes 4 consecutive rows.  With v = (row - r0) + shift, a slot's regular rows have
// v = vmin or vmin + DELTA; for a piece of LEN diagonals from d on, the slot loads the rows
// r0 + vmin + d + {0 .. LEN-1} and r0 + vmin + DELTA + d + {0 .. LEN-1} of X and every row multiplies
// with the one set or the other: the three rows of a grid point with three unknowns use the same rows of
// X, 6 loads for 12 products as in the plain case.
// The reference list may have up to 128 diagonals and the chunk's values need not fit one window: the
// list is worked through SEG diagonals at a time, and for each such pass the values of those diagonals
// of all regular rows are brought into LDS (row r at r * (SEG + 1): the slots' rows fall into different
// banks).  Pieces end at the passes' boundaries.  Odd rows read their values from memory.
template <typename T, int VEC, bool XCD_REMAP, int DELTA, int SEG>
__global__ __launch_bounds__(kWave) __attribute__((amdgpu_waves_per_eu(3)))
void spmm_block_shared_kernel(
    int32_t nrows, uint32_t num_chunks, uint32_t padded_chunks,
    const int32_t *__restrict__ stream_chunks, const int32_t *__restrict__ share_flag, int32_t want_flag,
    const int32_t *__restrict__ rowptr, uint32_t xcd_block,
    const T *__restrict__ vals, int64_t k, int64_t c0, const T *__restrict__ X, int64_t ldx, T *__restrict__ Y,
    int64_t ldy, T alpha, T beta, StreamPatterns pats, int32_t ncols)
{
    static_assert(DELTA == 2 || DELTA == 3, "two or three unknowns per grid point");
    static_assert(SEG == 32 || SEG == 64, "a pass is half a wavefront or a whole one");
    constexpr int CL = 8, kSlots = kWave / CL, R = kStreamRows / kSlots;
    constexpr int kStride = SEG + 1;
    constexpr int kBias = 64;                          // shifts are at least -64
    __shared__ T s_val[kStreamRows * kStride];

    const uint32_t id = !XCD_REMAP ? blockIdx.x
                        : xcd_block ? xcd_block_cyclic_id(blockIdx.x, xcd_block)
                                    : xcd_contiguous_id(blockIdx.x, padded_chunks);
    if (id >= num_chunks) return;
    const int lane = threadIdx.x;
    const int slot = lane / CL;
    const int l = lane % CL;
    const int64_t chunk = stream_chunks ? stream_chunks[id] : (int64_t)id;
    const int64_t row0 = chunk * kStreamRows;
    const int32_t flag = share_flag ? share_flag[chunk] : want_flag;       // wave-uniform
    const int32_t pat_begin = pats.pat_off[chunk];
    const ShareRows c = share_rows_setup(lane, nrows, row0, rowptr, pats.row_pat, 1, false);
    if (flag != want_flag) return;                                         // another kernel's chunk
    const int64_t col = c0 + (int64_t)l * VEC;
    const bool active = col < k;
    const int64_t col_ld = active ? col : c0;          // idle lanes stay for the LDS passes and load what lane 0 loads
    const uint32_t row_bytes = (uint32_t)(ldx * (int64_t)sizeof(T));
    // the stored list, diagonal t in lane t % 64 of pstar[t / 64] (every row adds its own shift)
    const int32_t *list = pats.pool + pat_begin + pattern_start(c.ref_pat);
    int32_t pstar[2];
    pstar[0] = lane < c.ref_len ? list[lane] : 0;
    pstar[1] = lane + kWave < c.ref_len ? list[lane + kWave] : 0;
    uint64_t m3[2], m2[2], m1[2];
    share_piece_masks<SEG>(pstar[0], c.ref_len, lane, m3[0], m2[0], m1[0]);
    share_piece_masks<SEG>(pstar[1], c.ref_len - kWave, lane, m3[1], m2[1], m1[1]);
    const uint64_t regular_rows = __builtin_amdgcn_ballot_w64(lane < kStreamRows && row0 + lane < nrows) & ~c.odd;

    // where this slot's rows stand and which of them use the second set of rows of X; a slot without a
    // regular row behaves like one whose rows all have v = 0
    const int r0 = slot * R;
    int32_t vmin = INT32_MAX;
    bool hi[R];
    {
        int32_t v[R];
#pragma unroll
        for (int pp = 0; pp < R; ++pp) {
            v[pp] = pp + pattern_shift(__shfl(c.my_pat, r0 + pp));
            if ((regular_rows >> (r0 + pp)) & 1) vmin = min(vmin, v[pp]);
        }
        if (vmin == INT32_MAX) vmin = 0;
#pragma unroll
        for (int pp = 0; pp < R; ++pp) hi[pp] = ((regular_rows >> (r0 + pp)) & 1) && v[pp] != vmin;
    }
    // row (row0 + r0 + vmin + d + q) of X = a wave-uniform address (row row0 - 64 + d + q) + this lane's fixed
    // offset.  Every row of X that a slot asks for on behalf of a regular row is the column of one of its
    // entries; the others (the second set of a slot whose rows all stand at vmin, slots with odd rows) may
    // lie outside X near the ends of the matrix: such chunks (`inside` false) clamp every row number.
    const uint32_t lane_off = (uint32_t)(r0 + vmin + kBias) * row_bytes + (uint32_t)(col_ld * (int64_t)sizeof(T));
    const char *x0 = reinterpret_cast<const char *>(X) + (row0 - kBias) * (int64_t)row_bytes;
    const int last = c.ref_len - 1;
    const int64_t d_min = __builtin_amdgcn_readlane(pstar[0], 0);
    const int64_t d_max = last < kWave ? __builtin_amdgcn_readlane(pstar[0], last) : __builtin_amdgcn_readlane(pstar[1], last - kWave);
    const int64_t lo_row = row0 + r0 + vmin + d_min, hi_row = row0 + r0 + vmin + d_max + DELTA;
    const bool inside = __builtin_amdgcn_ballot_w64(lo_row < 0 || hi_row > (int64_t)ncols - 1) == 0;   // uniform

    for (uint64_t left = c.odd; left != 0; left &= left - 1) {               // uniform
        const int row = (int)__builtin_ctzll(left);
        const int32_t rb = __builtin_amdgcn_readlane(c.my_rp, row), n = __builtin_amdgcn_readlane(c.my_len, row);
        const int32_t packed = __builtin_amdgcn_readlane(c.my_pat, row);
        share_odd_row<T, VEC, CL>(vals + rb, n, pats.pool + pat_begin + pattern_start(packed), row0 + row,
                                  row0 + row + pattern_shift(packed), slot, row / R == slot, active, col, k, X, ldx,
                                  Y, ldy, alpha, beta);
    }

    T acc[R][VEC];
#pragma unroll
    for (int pp = 0; pp < R; ++pp)
#pragma unroll
        for (int q = 0; q < VEC; ++q) acc[pp][q] = T(0);
    const T *my_val = s_val + r0 * kStride;            // this slot's rows in LDS
    // pieces of LEN diagonals of one pass: bit t of mask = a piece starts at diagonal t0 + t, which lane
    // t0 % 64 + t of `ps` holds
    auto run_class = [&](auto len_tag, auto inside_tag, uint64_t mask, int32_t ps, int lane0) {
        constexpr int LEN = decltype(len_tag)::value;
        constexpr bool kInside = decltype(inside_tag)::value;
        constexpr int NB = !kInside ? 2 : (LEN == 1 ? 4 : 3);   // pieces in flight (the rare clamped variant: fewer registers)
        // two arrays, so that the choice between the sets is one between two values, never an index into an array
        Pack<T, VEC> xlo[NB][LEN], xhi[NB][LEN];
        int tt[NB];
        auto fill = [&](int b) {
            tt[b] = (int)__builtin_ctzll(mask);
            mask &= mask - 1;
            const int32_t d = __builtin_amdgcn_readlane(ps, lane0 + tt[b]);
            const char *xb = x0 + (int64_t)d * (int64_t)row_bytes;            // uniform: scalar arithmetic
#pragma unroll
            for (int q = 0; q < LEN; ++q) {
                if constexpr (kInside) {
                    xlo[b][q] = *reinterpret_cast<const Pack<T, VEC> *>(xb + (int64_t)q * (int64_t)row_bytes + lane_off);
                    xhi[b][q] = *reinterpret_cast<const Pack<T, VEC> *>(xb + (int64_t)(DELTA + q) * (int64_t)row_bytes + lane_off);
                } else {
                    const int64_t top = (int64_t)ncols - 1;
                    int64_t r = row0 + r0 + vmin + d + q, r2 = r + DELTA;
                    r = r < 0 ? 0 : (r > top ? top : r);
                    r2 = r2 < 0 ? 0 : (r2 > top ? top : r2);
                    xlo[b][q] = *reinterpret_cast<const Pack<T, VEC> *>(X + r * ldx + col_ld);
                    xhi[b][q] = *reinterpret_cast<const Pack<T, VEC> *>(X + r2 * ldx + col_ld);
                }
            }
        };
        auto use = [&](int b) {
            T v[LEN][R];
#pragma unroll
            for (int e = 0; e < LEN; ++e)
#pragma unroll
                for (int pp = 0; pp < R; ++pp) v[e][pp] = my_val[pp * kStride + tt[b] + e];
#pragma unroll
            for (int e = 0; e < LEN; ++e)
#pragma unroll
                for (int pp = 0; pp < R; ++pp)
#pragma unroll
                    for (int q = 0; q < VEC; ++q)
                        acc[pp][q] = fused_madd(v[e][pp], hi[pp] ? xhi[b][e].v[q] : xlo[b][e].v[q], acc[pp][q]);
        };
        int left = __popcll(mask);                         // pieces not yet asked for
        if (left >= NB) {
#pragma unroll
            for (int b = 0; b < NB; ++b) fill(b);
            left -= NB;
#pragma unroll 1
            while (left >= NB) {                           // steady state: every piece multiplied out is replaced
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    use(b);
                    __builtin_amdgcn_sched_barrier(0);     // the refill stays below the products it replaces
                    fill(b);
                    __builtin_amdgcn_sched_barrier(0);
                }
                left -= NB;
            }
#pragma unroll
            for (int b = 0; b < NB; ++b) use(b);
            __builtin_amdgcn_sched_barrier(0);
        }
        // fewer than NB pieces are left
#pragma unroll
        for (int b = 0; b < NB - 1; ++b)
            if (b < left) fill(b);
#pragma unroll
        for (int b = 0; b < NB - 1; ++b)
            if (b < left) use(b);
    };

    constexpr int kRowsPerStep = kWave / SEG;          // rows of the chunk one load instruction covers
#pragma unroll 1
    for (int t0 = 0; t0 < c.ref_len; t0 += SEG) {                            // uniform: one pass per SEG diagonals
        // the values of diagonals t0 .. t0 + SEG - 1 of every regular row; the others' places hold zeros
        const int j = lane % SEG;
        T staged[kStreamRows / kRowsPerStep];
#pragma unroll
        for (int i = 0; i < kStreamRows / kRowsPerStep; ++i) {
            int row = i;
            int32_t rp = __builtin_amdgcn_readlane(c.my_rp, i * kRowsPerStep);
            if constexpr (kRowsPerStep == 2) {
                const int32_t rp_b = __builtin_amdgcn_readlane(c.my_rp, 2 * i + 1);
                row = 2 * i + lane / SEG;
                rp = lane < SEG ? rp : rp_b;
            }
            const bool have = ((regular_rows >> row) & 1) && t0 + j < c.ref_len;
            staged[i] = have ? vals[(int64_t)rp + t0 + j] : T(0);
        }
#pragma unroll
        for (int i = 0; i < kStreamRows / kRowsPerStep; ++i)
            s_val[(i * kRowsPerStep + lane / SEG) * kStride + j] = staged[i];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        const int half = t0 / kWave, lane0 = t0 % kWave;                      // uniform
        const uint64_t seg_mask = SEG == kWave ? ~0ull : 0xffffffffull;
        const uint64_t p3 = ((half ? m3[1] : m3[0]) >> lane0) & seg_mask;
        const uint64_t p2 = ((half ? m2[1] : m2[0]) >> lane0) & seg_mask;
        const uint64_t p1 = ((half ? m1[1] : m1[0]) >> lane0) & seg_mask;
        const int32_t ps = half ? pstar[1] : pstar[0];
        if (inside) {
            if (p3) run_class(std::integral_constant<int, 3>(), std::true_type(), p3, ps, lane0);
            if (p2) run_class(std::integral_constant<int, 2>(), std::true_type(), p2, ps, lane0);
            if (p1) run_class(std::integral_constant<int, 1>(), std::true_type(), p1, ps, lane0);
        } else {
            if (p3) run_class(std::integral_constant<int, 3>(), std::false_type(), p3, ps, lane0);
            if (p2) run_class(std::integral_constant<int, 2>(), std::false_type(), p2, ps, lane0);
            if (p1) run_class(std::integral_constant<int, 1>(), std::false_type(), p1, ps, lane0);
        }
        // the next pass overwrites what this one read
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    if (!active) return;
#pragma unroll
    for (int pp = 0; pp < R; ++pp)
        if ((regular_rows >> (r0 + pp)) & 1) store_row<T, VEC>(Y + (row0 + r0 + pp) * ldy, acc[pp], col, k, alpha, beta);
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
