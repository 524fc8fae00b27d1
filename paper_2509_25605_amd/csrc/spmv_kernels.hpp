// SpMV kernels for gfx950: y = alpha*A*x + beta*y with A in CSR (Section 6.2),
// rows walked with the CSR loop nest of Section 4.2.
//
//  * spmv_stream_kernel: one wavefront per 64/G consecutive rows of a stream chunk
//    (32 consecutive rows; G = 2, 4, 8, 16 lanes per row by the chunk's class).
//    The rows' entries are one contiguous range of the value / column arrays: the
//    wavefront streams it with 16-byte non-temporal loads into LDS (16-bit column
//    offsets instead of 32-bit columns where the analysis built them), then a
//    group of G lanes per row walks the row out of LDS and gathers x.
//    Consecutive rows sit in consecutive lane groups, so for banded matrices
//    (stencils, FEM) every gather instruction reads a nearly contiguous piece of x.
//  * spmv_short_kernel: one launch covers bins 0..8 of the row partition.  A
//    group of G = 2^(bin-1) lanes owns a row, the lanes stride the row's
//    entries (the ThreadVector level of Section 4.2 "Loop translation", with
//    the vector length chosen per row instead of per matrix), a DPP reduction
//    folds the group and one lane stores y[i] (the `single` of Section 4.2
//    "Synchronizations").
//  * spmv_long_tile_kernel + spmv_long_fixup_kernel: rows of bin 9 are cut into
//    equal tiles of entries; a workgroup reduces one tile through LDS and a
//    second pass adds a row's tile sums in tile order, so every y[i] has one
//    writer and the result does not depend on scheduling.
//  * spmv_ldsblock_kernel + spmv_ldsblock_combine_kernel: rows above LAPIS_HUGE_ROW
//    entries, cut at column blocks of x that fit LDS; their gathers are LDS reads.
#pragma once
#include <type_traits>

#include "device_utils.hpp"

namespace lapis {

constexpr int kShortBins = 9;  // bins 0..8 are handled by the short-row kernel

// Rows handled per lane group in one workgroup pass, per bin.  More rows per
// group = more independent loads in flight per lane.
__host__ __device__ constexpr int short_rows_per_group(int bin)
{
    return bin == 0 ? 1 : bin <= 3 ? 4 : bin <= 5 ? 4 : bin <= 7 ? 4 : 1;
}
__host__ __device__ constexpr int short_group_size(int bin)
{
    return bin == 0 ? 1 : bin >= 8 ? 64 : (1 << (bin - 1));
}
__host__ __device__ constexpr int short_rows_per_block(int bin)
{
    return (kBlock / short_group_size(bin)) * short_rows_per_group(bin);
}

// Workgroups of bin b occupy hardware ids [block_begin[b], block_begin[b+1]); every bin's count
// is padded to a multiple of the XCD count, so inside a bin hardware id h runs on XCD h % 8 and
// xcd_contiguous_id gives each XCD one contiguous stretch of the bin's row list.
struct ShortPlan {
    int32_t bin_begin[kShortBins];        // first position of bin b in row_perm
    int32_t bin_count[kShortBins];        // rows in bin b
    uint32_t block_begin[kShortBins + 1]; // padded workgroup ranges per bin
    uint32_t num_blocks;                  // block_begin[kShortBins] = grid size
};

template <typename T>
__device__ __forceinline__ void store_result(T *__restrict__ y, int32_t row, T s, T alpha, T beta)
{
    y[row] = (beta == T(0)) ? alpha * s : alpha * s + beta * y[row];
}

// Rows with at most G entries: a single pass, U rows per group.
template <typename T, int G, int U>
__device__ __forceinline__ void short_rows(uint32_t local_block, int32_t begin, int32_t count,
                                           const int32_t *__restrict__ row_perm,
                                           const int32_t *__restrict__ row_begin,
                                           const int32_t *__restrict__ row_end,
                                           const int32_t *__restrict__ colidx,
                                           const T *__restrict__ vals, const T *__restrict__ x,
                                           T *__restrict__ y, T alpha, T beta)
{
    constexpr int kGroups = kBlock / G;
    const int group = threadIdx.x / G;
    const int lane = threadIdx.x % G;
    const int64_t base = (int64_t)local_block * (kGroups * U);

    int32_t row[U];
    int32_t jb[U], je[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t idx = base + u * kGroups + group;
        row[u] = (idx < count) ? row_perm[begin + idx] : -1;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        jb[u] = (row[u] >= 0) ? row_begin[row[u]] : 0;
        je[u] = (row[u] >= 0) ? row_end[row[u]] : 0;
    }
    int32_t c[U];
    T v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t j = (int64_t)jb[u] + lane;
        const bool in = j < je[u];
        c[u] = in ? load_stream(colidx + j) : -1;
        v[u] = in ? load_stream(vals + j) : T(0);
    }
    T s[U];
#pragma unroll
    for (int u = 0; u < U; ++u) s[u] = (c[u] >= 0) ? v[u] * x[c[u]] : T(0);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        s[u] = group_sum<G>(s[u]);
        if (lane == G - 1 && row[u] >= 0) store_result(y, row[u], s[u], alpha, beta);
    }
}

// Rows with 65 .. long-threshold entries: one wavefront walks the row.
template <typename T>
__device__ __forceinline__ void wave_rows(uint32_t local_block, int32_t begin, int32_t count,
                                          const int32_t *__restrict__ row_perm,
                                          const int32_t *__restrict__ row_begin,
                                          const int32_t *__restrict__ row_end,
                                          const int32_t *__restrict__ colidx,
                                          const T *__restrict__ vals, const T *__restrict__ x,
                                          T *__restrict__ y, T alpha, T beta)
{
    const int wave = threadIdx.x / kWave;
    const int lane = threadIdx.x % kWave;
    const int64_t idx = (int64_t)local_block * kWavesPerBlock + wave;
    const int32_t row = (idx < count) ? row_perm[begin + idx] : -1;
    const int64_t jb = (row >= 0) ? row_begin[row] : 0;
    const int64_t je = (row >= 0) ? row_end[row] : 0;
    T s0 = T(0), s1 = T(0), s2 = T(0), s3 = T(0);
    int64_t j = jb + lane;
    for (; j + 3 * kWave < je; j += 4 * kWave) {
        const int32_t c0 = load_stream(colidx + j), c1 = load_stream(colidx + j + kWave);
        const int32_t c2 = load_stream(colidx + j + 2 * kWave), c3 = load_stream(colidx + j + 3 * kWave);
        const T v0 = load_stream(vals + j), v1 = load_stream(vals + j + kWave);
        const T v2 = load_stream(vals + j + 2 * kWave), v3 = load_stream(vals + j + 3 * kWave);
        s0 += v0 * x[c0];
        s1 += v1 * x[c1];
        s2 += v2 * x[c2];
        s3 += v3 * x[c3];
    }
    for (; j < je; j += kWave) s0 += load_stream(vals + j) * x[load_stream(colidx + j)];
    T s = group_sum<kWave>((s0 + s1) + (s2 + s3));
    if (lane == kWave - 1 && row >= 0) store_result(y, row, s, alpha, beta);
}

// row_begin[i] / row_end[i] delimit row i's entries: (rowptr, rowptr + 1) for the rows of the
// matrix, the cut table for virtual rows.
template <typename T, bool XCD_REMAP>
__global__ __launch_bounds__(kBlock) void spmv_short_kernel(
    ShortPlan plan, const int32_t *__restrict__ row_perm, const int32_t *__restrict__ row_begin,
    const int32_t *__restrict__ row_end, const int32_t *__restrict__ colidx,
    const T *__restrict__ vals, const T *__restrict__ x, T *__restrict__ y, T alpha, T beta)
{
    const uint32_t hw = blockIdx.x;
    int bin = 0;
    while (hw >= plan.block_begin[bin + 1]) ++bin;  // uniform over the workgroup
    const uint32_t in_bin = hw - plan.block_begin[bin];
    const uint32_t padded = plan.block_begin[bin + 1] - plan.block_begin[bin];
    const uint32_t local = XCD_REMAP ? xcd_contiguous_id(in_bin, padded) : in_bin;
    const int32_t begin = plan.bin_begin[bin], count = plan.bin_count[bin];
    // workgroups past the bin's last row (padding) find idx >= count everywhere and do nothing
#define LAPIS_SHORT_CASE(B)                                                                     \
    case B:                                                                                     \
        short_rows<T, short_group_size(B), short_rows_per_group(B)>(local, begin, count,        \
            row_perm, row_begin, row_end, colidx, vals, x, y, alpha, beta);                     \
        break;
    switch (bin) {
    case 0: {  // rows without entries: y = beta*y
        const int64_t idx = (int64_t)local * kBlock + threadIdx.x;
        if (idx < count) store_result(y, row_perm[begin + idx], T(0), alpha, beta);
        break;
    }
        LAPIS_SHORT_CASE(1)
        LAPIS_SHORT_CASE(2)
        LAPIS_SHORT_CASE(3)
        LAPIS_SHORT_CASE(4)
        LAPIS_SHORT_CASE(5)
        LAPIS_SHORT_CASE(6)
        LAPIS_SHORT_CASE(7)
    default:
        wave_rows<T>(local, begin, count, row_perm, row_begin, row_end, colidx, vals, x, y, alpha, beta);
        break;
    }
#undef LAPIS_SHORT_CASE
}

// ---- stream chunks ----------------------------------------------------------
constexpr int kStreamRows = 32;                      // rows per chunk
constexpr int kStreamClasses = 4;                    // chunk classes 1..4: 2, 4, 8, 16 lanes per row
constexpr int kStreamWindow = 1024;                  // entries staged in LDS at a time
constexpr int kStreamUnroll = 16;                    // gathers in flight per lane and batch

template <typename T> struct StreamVec;
template <> struct StreamVec<double> { typedef double type __attribute__((ext_vector_type(2))); };
template <> struct StreamVec<float> { typedef float type __attribute__((ext_vector_type(4))); };
typedef int32_t int4v __attribute__((ext_vector_type(4)));

typedef uint16_t ushort8v __attribute__((ext_vector_type(8)));

// Where a window's column indices come from: the matrix's 32-bit colidx, or (cbase >= 0) the
// 16-bit offsets col16 from the chunk's smallest column cbase, which the analysis builds for
// chunks whose columns span less than 2^16.  Both pointers are already advanced to the window.
struct StreamCols {
    const int32_t *__restrict__ c32;
    const uint16_t *__restrict__ c16;     // window start a multiple of 8 entries (16 bytes); padded past nnz
    int32_t cbase;
    const int32_t *tab;                   // LDS: the chunk's frame table (framed chunks only)
};

// How a chunk's columns are stored: 32-bit colidx; 16-bit offsets from the chunk's smallest
// column (chunk_base >= 0); or 16-bit codes (slot << 11) | (column & 2047) with a per-chunk table
// of up to 32 frames of 2048 columns (chunk_base == kChunkFramed).
constexpr int kCols32 = 0, kColsNarrow = 1, kColsFramed = 2, kColsEither = 3;   // kColsEither: narrow or framed, per chunk
// A patterned chunk needs no columns per entry at all: equal rows of the chunk share one list
// of diagonals (column - row) in the chunk's pattern table, and a row only knows where its list
// starts.  kColsPattern: every chunk of the launch is patterned; kColsPatternOr16: patterned, or
// else narrow or framed.  kColsNone: a window of values only.
constexpr int kColsPattern = 4, kColsPatternOr16 = 5, kColsNone = -1;
constexpr int kPatternTable = 512;                   // diagonals in a chunk's pattern table at most
constexpr int32_t kChunkFramed = -2;
constexpr int kFrameShift = 11, kFrameSlots = 32;
constexpr int32_t kFrameMask = (1 << kFrameShift) - 1;

__device__ __forceinline__ int32_t framed_column(const int32_t *tab, uint16_t code)
{
    return (tab[code >> kFrameShift] << kFrameShift) | ((int32_t)code & kFrameMask);
}

// Copy the first n_vec (a multiple of 4, <= kStreamWindow) entries of the window to LDS with
// NC column loads (16 bytes, or 8 bytes of 16-bit offsets) and NV 16-byte value loads per lane.
// Lanes past the end repeat the last group: same address, same data, no extra memory traffic
// and no divergent control flow.
template <typename T, int NC, int NV, int KIND, typename IDX>
__device__ __forceinline__ void stream_fill(const StreamCols cols, const T *__restrict__ vw,
                                            int lane, int n_vec, IDX *s_col, T *s_val)
{
    constexpr bool C16 = KIND != kCols32 && KIND != kColsNone;
    constexpr bool kRaw16 = sizeof(IDX) == 2;       // LDS keeps the 16-bit offsets as they are
    static_assert(!kRaw16 || KIND == kColsNarrow, "a 16-bit LDS window needs 16-bit offsets in memory");
    typedef typename StreamVec<T>::type vec_t;
    constexpr int kPerVec = 16 / sizeof(T);          // values per 16-byte load
    const int last_c = n_vec - 4;
    const int last_v = n_vec - kPerVec;
    constexpr int NC8 = (NC + 1) / 2;               // 16-byte loads of 8 offsets cover 512 entries
    const int last_c8 = ((n_vec + 7) & ~7) - 8;
    int4v cq[C16 ? 1 : NC];
    ushort8v cs[C16 ? NC8 : 1];
    vec_t vq[NV];
    if constexpr (C16) {
#pragma unroll
        for (int i = 0; i < NC8; ++i) {
            int idx = i * (kWave * 8) + lane * 8;
            idx = idx < last_c8 ? idx : last_c8;
            cs[i] = __builtin_nontemporal_load(reinterpret_cast<const ushort8v *>(cols.c16 + idx));
        }
    } else if constexpr (KIND != kColsNone) {
#pragma unroll
        for (int i = 0; i < NC; ++i) {
            int idx = i * (kWave * 4) + lane * 4;
            idx = idx < last_c ? idx : last_c;
            cq[i] = __builtin_nontemporal_load(reinterpret_cast<const int4v *>(cols.c32 + idx));
        }
    }
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        int idx = i * (kWave * kPerVec) + lane * kPerVec;
        idx = idx < last_v ? idx : last_v;
        vq[i] = __builtin_nontemporal_load(reinterpret_cast<const vec_t *>(vw + idx));
    }
    if constexpr (C16) {
#pragma unroll
        for (int i = 0; i < NC8; ++i) {
            int idx = i * (kWave * 8) + lane * 8;
            idx = idx < last_c8 ? idx : last_c8;
            if constexpr (kRaw16) {
                *reinterpret_cast<ushort8v *>(s_col + idx) = cs[i];
                continue;
            }
            int4v a, b;
            if constexpr (KIND == kColsFramed) {
                a.x = framed_column(cols.tab, cs[i].s0); a.y = framed_column(cols.tab, cs[i].s1);
                a.z = framed_column(cols.tab, cs[i].s2); a.w = framed_column(cols.tab, cs[i].s3);
                b.x = framed_column(cols.tab, cs[i].s4); b.y = framed_column(cols.tab, cs[i].s5);
                b.z = framed_column(cols.tab, cs[i].s6); b.w = framed_column(cols.tab, cs[i].s7);
            } else {
                a.x = cols.cbase + (int32_t)cs[i].s0; a.y = cols.cbase + (int32_t)cs[i].s1;
                a.z = cols.cbase + (int32_t)cs[i].s2; a.w = cols.cbase + (int32_t)cs[i].s3;
                b.x = cols.cbase + (int32_t)cs[i].s4; b.y = cols.cbase + (int32_t)cs[i].s5;
                b.z = cols.cbase + (int32_t)cs[i].s6; b.w = cols.cbase + (int32_t)cs[i].s7;
            }
            *reinterpret_cast<int4v *>(s_col + idx) = a;
            *reinterpret_cast<int4v *>(s_col + idx + 4) = b;
        }
    } else if constexpr (KIND != kColsNone) {
#pragma unroll
        for (int i = 0; i < NC; ++i) {
            int idx = i * (kWave * 4) + lane * 4;
            idx = idx < last_c ? idx : last_c;
            *reinterpret_cast<int4v *>(s_col + idx) = cq[i];
        }
    }
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        int idx = i * (kWave * kPerVec) + lane * kPerVec;
        idx = idx < last_v ? idx : last_v;
        *reinterpret_cast<vec_t *>(s_val + idx) = vq[i];
    }
}

// NC column loads cover NC*256 entries; the value loads needed for n_vec entries are either
// NC*R or NC*R - 1 (R = value loads per 256 entries: 2 for double, 1 for float).
template <typename T, int NC, int KIND, typename IDX>
__device__ __forceinline__ void stream_fill_pick(const StreamCols cols, const T *__restrict__ vw,
                                                 int lane, int n_vec, IDX *s_col, T *s_val)
{
    constexpr int kPerLoad = kWave * (16 / (int)sizeof(T));   // entries per value load instruction
    constexpr int kFull = NC * (kWave * 4) / kPerLoad;
    if constexpr (kFull > 1 && kPerLoad < kWave * 4) {
        if (n_vec <= (kFull - 1) * kPerLoad) {
            stream_fill<T, NC, kFull - 1, KIND, IDX>(cols, vw, lane, n_vec, s_col, s_val);
            return;
        }
    }
    stream_fill<T, NC, kFull, KIND, IDX>(cols, vw, lane, n_vec, s_col, s_val);
}

template <typename T, int KIND, typename IDX>
__device__ __forceinline__ void stream_fill_by_size(const StreamCols cols, const T *__restrict__ vw,
                                                    int lane, int n_vec, IDX *s_col, T *s_val)
{
    if (n_vec > 3 * kWave * 4) stream_fill_pick<T, 4, KIND, IDX>(cols, vw, lane, n_vec, s_col, s_val);
    else if (n_vec > 2 * kWave * 4) stream_fill_pick<T, 3, KIND, IDX>(cols, vw, lane, n_vec, s_col, s_val);
    else if (n_vec > kWave * 4) stream_fill_pick<T, 2, KIND, IDX>(cols, vw, lane, n_vec, s_col, s_val);
    else if (n_vec > 0) stream_fill_pick<T, 1, KIND, IDX>(cols, vw, lane, n_vec, s_col, s_val);
}

// Stage entries [w0, w1) of the matrix (w0 a multiple of 8, w1 - w0 <= kStreamWindow) in LDS:
// vector loads up to nnz4 (= nnz rounded down to a multiple of 4), the matrix's last nnz % 4
// entries one by one.  cbase >= 0: the columns are cbase + col16[j], else colidx[j] (col16 may
// then be null).  Ends with a wavefront-level fence so every lane may read what others wrote.
// With a 16-bit LDS window (IDX = uint16_t) the offsets are staged as they are and cbase must be >= 0.
// cbase == kChunkFramed: the codes are expanded through the chunk's frame table s_tab (LDS, filled
// and fenced by the caller).
template <typename T, typename IDX>
__device__ __forceinline__ void stream_window_to_lds(const int32_t *__restrict__ colidx,
                                                     const uint16_t *__restrict__ col16, int32_t cbase,
                                                     const int32_t *s_tab,
                                                     const T *__restrict__ vals, int32_t w0, int32_t w1,
                                                     int32_t nnz4, int lane, IDX *s_col, T *s_val)
{
    constexpr bool kRaw16 = sizeof(IDX) == 2;
    const int32_t vec_end = w1 < nnz4 ? ((w1 + 3) & ~3) : nnz4;   // vector loads stop here
    const int n_vec = vec_end > w0 ? vec_end - w0 : 0;
    const T *__restrict__ vw = vals + w0;
    if constexpr (kRaw16) {
        stream_fill_by_size<T, kColsNarrow, IDX>(StreamCols{nullptr, col16 + w0, cbase, nullptr}, vw, lane, n_vec, s_col, s_val);
    } else {
        if (cbase >= 0) stream_fill_by_size<T, kColsNarrow, IDX>(StreamCols{nullptr, col16 + w0, cbase, nullptr}, vw, lane, n_vec, s_col, s_val);
        else if (cbase == kChunkFramed) stream_fill_by_size<T, kColsFramed, IDX>(StreamCols{nullptr, col16 + w0, 0, s_tab}, vw, lane, n_vec, s_col, s_val);
        else stream_fill_by_size<T, kCols32, IDX>(StreamCols{colidx + w0, nullptr, 0, nullptr}, vw, lane, n_vec, s_col, s_val);
    }
    if (w0 + n_vec < w1) {                              // the matrix's last nnz % 4 entries
        const int32_t j = w0 + n_vec + lane;
        if (j < w1) {
            if constexpr (kRaw16) s_col[j - w0] = col16[j];
            else s_col[j - w0] = cbase >= 0 ? cbase + (int32_t)col16[j]
                                 : cbase == kChunkFramed ? framed_column(s_tab, col16[j]) : colidx[j];
            s_val[j - w0] = vals[j];
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// The values alone of entries [w0, w1) into LDS (patterned chunks keep no columns per entry);
// same alignment rules and the same closing fence as stream_window_to_lds.
template <typename T>
__device__ __forceinline__ void stream_values_to_lds(const T *__restrict__ vals, int32_t w0, int32_t w1,
                                                     int32_t nnz4, int lane, T *s_val)
{
    const int32_t vec_end = w1 < nnz4 ? ((w1 + 3) & ~3) : nnz4;
    const int n_vec = vec_end > w0 ? vec_end - w0 : 0;
    stream_fill_by_size<T, kColsNone, int32_t>(StreamCols{nullptr, nullptr, 0, nullptr}, vals + w0, lane, n_vec,
                                               nullptr, s_val);
    if (w0 + n_vec < w1) {
        const int32_t j = w0 + n_vec + lane;
        if (j < w1) s_val[j - w0] = vals[j];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// The frame table of a framed chunk into LDS (32 ints per wavefront), fenced for the wavefront.
__device__ __forceinline__ void load_frame_table(const int32_t *__restrict__ frame_table, int64_t chunk,
                                                 int32_t cbase, int lane, int32_t *s_tab)
{
    if (cbase == kChunkFramed) {
        if (lane < kFrameSlots) s_tab[lane] = frame_table[chunk * kFrameSlots + lane];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
}

__device__ __forceinline__ double fused_madd(double a, double b, double c) { return __builtin_fma(a, b, c); }
__device__ __forceinline__ float fused_madd(float a, float b, float c) { return __builtin_fmaf(a, b, c); }

// B entries of this lane's share of a row: (column, value) pairs out of LDS, the B gathers of x
// issued back to back, then the multiply-adds.  The first W of the B entries exist in every lane of
// the wavefront (the caller knows the shortest share): they need no clamp and no select and use
// FMAs.  For the others, lanes with fewer than u0 + B entries repeat their last entry and discard
// the product (no divergent control flow).
// x is already advanced by the chunk's smallest column when the window holds 16-bit offsets.
// RAW == kColsFramed: the window holds raw frame codes, expanded here through the table `tab`;
// RAW == kColsEither: offsets from cbase if cbase >= 0 (wave-uniform), else frame codes.
template <typename T, int B, int W, int G, typename IDX, int RAW>
__device__ __forceinline__ T stream_batch(const IDX *sc, const T *sv, int u0, int my_n, int last_u,
                                          const T *__restrict__ x, const int32_t *tab, int32_t cbase, T s)
{
    static_assert(W >= 0 && W <= B, "W counts leading entries of the batch");
    int32_t cc[B];
    T vv[B], xx[B];
#pragma unroll
    for (int t = 0; t < B; ++t) {
        const int u = (t < W ? u0 + t : (u0 + t < last_u ? u0 + t : last_u)) * G;
        cc[t] = (int32_t)sc[u];
        vv[t] = sv[u];
    }
    if constexpr (RAW == kColsFramed) {
#pragma unroll
        for (int t = 0; t < B; ++t) cc[t] = framed_column(tab, (uint16_t)cc[t]);
    } else if constexpr (RAW == kColsEither) {
        if (cbase >= 0) {
#pragma unroll
            for (int t = 0; t < B; ++t) cc[t] += cbase;
        } else {
#pragma unroll
            for (int t = 0; t < B; ++t) cc[t] = framed_column(tab, (uint16_t)cc[t]);
        }
    }
#pragma unroll
    for (int t = 0; t < B; ++t) xx[t] = x[cc[t]];
#pragma unroll
    for (int t = 0; t < B; ++t) {
        if (t < W) s = fused_madd(vv[t], xx[t], s);
        else s += (u0 + t < my_n) ? vv[t] * xx[t] : T(0);
    }
    return s;
}

// The batch of B with as many unconditional leading entries as the shortest share allows:
// all B, all but the last two (shares in a wavefront usually differ by at most one), or none.
template <typename T, int B, int G, typename IDX, int RAW>
__device__ __forceinline__ T stream_batch_pick(const IDX *sc, const T *sv, int u0, int my_n, int last_u,
                                               int shortest, const T *__restrict__ x, const int32_t *tab,
                                               int32_t cbase, T s)
{
    if (shortest - u0 >= B) return stream_batch<T, B, B, G, IDX, RAW>(sc, sv, u0, my_n, last_u, x, tab, cbase, s);
    if constexpr (B > 2) {
        if (shortest - u0 >= B - 2)
            return stream_batch<T, B, B - 2, G, IDX, RAW>(sc, sv, u0, my_n, last_u, x, tab, cbase, s);
    }
    return stream_batch<T, B, 0, G, IDX, RAW>(sc, sv, u0, my_n, last_u, x, tab, cbase, s);
}

// One lane's share of a row out of a staged window: my_n entries (<= 0: none) at sc[u * G] /
// sv[u * G], u = 0 .. my_n - 1, in batches of UNR gathers.  The last batch is cut to the longest
// share in the wavefront (rounded up to even), so rows of 27 entries issue 14 gathers per lane,
// not 16.  All lanes of the wavefront must call this together.
template <typename T, int G, typename IDX, int RAW, int UNR>
__device__ __forceinline__ T stream_share(const IDX *sc, const T *sv, int my_n, const T *__restrict__ xb,
                                          const int32_t *s_tab, int32_t cbase, T s)
{
    static_assert(UNR == 16, "the last-batch switch below enumerates even sizes up to 16");
    const int last_u = my_n > 0 ? my_n - 1 : 0;
    int rem = wave_max_nonneg(my_n > 0 ? my_n : 0);
    const int shortest = kStreamWindow - wave_max_nonneg(kStreamWindow - (my_n > 0 ? my_n : 0));   // uniform
    int u0 = 0;
#pragma unroll 1
    for (; rem > UNR; rem -= UNR, u0 += UNR) s = stream_batch_pick<T, UNR, G, IDX, RAW>(sc, sv, u0, my_n, last_u, shortest, xb, s_tab, cbase, s);
    switch ((rem + 1) / 2) {
    case 0: break;
    case 1: s = stream_batch_pick<T, 2, G, IDX, RAW>(sc, sv, u0, my_n, last_u, shortest, xb, s_tab, cbase, s); break;
    case 2: s = stream_batch_pick<T, 4, G, IDX, RAW>(sc, sv, u0, my_n, last_u, shortest, xb, s_tab, cbase, s); break;
    case 3: s = stream_batch_pick<T, 6, G, IDX, RAW>(sc, sv, u0, my_n, last_u, shortest, xb, s_tab, cbase, s); break;
    case 4: s = stream_batch_pick<T, 8, G, IDX, RAW>(sc, sv, u0, my_n, last_u, shortest, xb, s_tab, cbase, s); break;
    case 5: s = stream_batch_pick<T, 10, G, IDX, RAW>(sc, sv, u0, my_n, last_u, shortest, xb, s_tab, cbase, s); break;
    case 6: s = stream_batch_pick<T, 12, G, IDX, RAW>(sc, sv, u0, my_n, last_u, shortest, xb, s_tab, cbase, s); break;
    case 7: s = stream_batch_pick<T, 14, G, IDX, RAW>(sc, sv, u0, my_n, last_u, shortest, xb, s_tab, cbase, s); break;
    default: s = stream_batch_pick<T, UNR, G, IDX, RAW>(sc, sv, u0, my_n, last_u, shortest, xb, s_tab, cbase, s); break;
    }
    return s;
}

// One wavefront (= one workgroup) per 64/G consecutive rows of a stream chunk of the class with
// G lanes per row (G = 2, 4, 8, 16: a chunk of 32 rows is shared by G/2 wavefronts).
// stream_chunks lists the chunks of that class; nullptr means every chunk of the matrix.
// colidx and vals must be 16-byte aligned.  nnz4 = nnz rounded down to a multiple of 4:
// 16-byte loads never reach past it, the last nnz % 4 entries of the matrix are fetched one by one.
// RAW == kColsNarrow: every chunk of this launch is narrow (chunk_base >= 0); RAW == kColsFramed:
// every chunk is framed.  The LDS window then keeps the 2-byte offsets / codes as they are (10
// instead of 12 KB per wavefront with doubles: more wavefronts per CU) and they are expanded
// when x is gathered.  RAW == kColsEither: every chunk is one or the other.  RAW == kCols32: any
// mix, 32-bit columns in the window.  RAW == kColsPattern: every chunk is patterned
// (pat_off[chunk + 1] > pat_off[chunk]): only the values are streamed, the chunk's table of
// diagonals (pool + pat_off[chunk]) takes the window's place in LDS and row_pat[row] says where
// the row's list starts in it and by how much it is shifted.  RAW == kColsPatternOr16: patterned, else narrow or framed.
struct StreamPatterns {
    const int32_t *__restrict__ pat_off;     // [num_chunks + 1]
    const uint16_t *__restrict__ row_pat;    // [nrows] start of the row's list in its chunk's table | shift << 9
    const int32_t *__restrict__ pool;
};
// row_pat[i] packs where the row's list starts in the chunk's table (bits 0..8) and the shift
// (-64..63, bits 9..15) that turns the stored list into the row's own:
// column k of row i = i + shift + table[start + k].
__device__ __forceinline__ int32_t pattern_start(int32_t packed) { return packed & 511; }
__device__ __forceinline__ int32_t pattern_shift(int32_t packed) { return (int32_t)(int16_t)(uint16_t)packed >> 9; }

template <typename T, int G, bool XCD_REMAP, int RAW = kCols32, int UNR = kStreamUnroll, int GW = 1>  // UNR must be 16
__global__ __launch_bounds__(kWave * GW) void spmv_stream_kernel(
    int32_t nrows, int32_t nnz, uint32_t num_waves, uint32_t padded_waves,
    const int32_t *__restrict__ stream_chunks, const int32_t *__restrict__ rowptr,
    const int32_t *__restrict__ colidx, const int32_t *__restrict__ chunk_base,
    const int32_t *__restrict__ frame_table, const uint16_t *__restrict__ col16, const StreamPatterns pats,
    const T *__restrict__ vals, const T *__restrict__ x, T *__restrict__ y, T alpha, T beta)
{
    constexpr int kRowsPerWave = kWave / G;
    constexpr int kWavesPerChunk = kStreamRows / kRowsPerWave;
    static_assert(G >= 2 && G <= 16 && kWavesPerChunk * kRowsPerWave == kStreamRows, "G must be 2, 4, 8 or 16");
    constexpr bool kHasPatterns = RAW == kColsPattern || RAW == kColsPatternOr16;
    constexpr int kShareMode = RAW == kColsPatternOr16 ? kColsEither : RAW;       // how the 16-bit window is read
    typedef typename std::conditional<RAW != kCols32, uint16_t, int32_t>::type idx_t;
    static_assert(kPatternTable * sizeof(int32_t) == kStreamWindow * sizeof(uint16_t), "the table takes the window's place");
    // GW > 1: GW wavefronts with consecutive ids (the wavefronts of one chunk, or of neighbouring
    // chunks) form one workgroup.  They share nothing but the CU and its L1, which pays when every
    // gather touches a cache line of its own (they gather from the same neighbourhood of x);
    // padded_waves then counts workgroups.
    constexpr int kGroup = GW;
    __shared__ __attribute__((aligned(16))) T s_val_all[kGroup][kStreamWindow];
    __shared__ __attribute__((aligned(16))) idx_t s_col_all[kGroup][kStreamWindow];
    __shared__ int32_t s_tab_all[kGroup][(RAW == kColsNarrow || RAW == kColsPattern) ? 1 : kFrameSlots];
    const int wave_in_group = GW > 1 ? threadIdx.x / kWave : 0;
    T *s_val = s_val_all[wave_in_group];
    idx_t *s_col = s_col_all[wave_in_group];
    int32_t *s_tab = s_tab_all[wave_in_group];
    int32_t *s_pat = reinterpret_cast<int32_t *>(s_col);

    const uint32_t id = (XCD_REMAP ? xcd_contiguous_id(blockIdx.x, padded_waves) : blockIdx.x) * kGroup + wave_in_group;
    if (id >= num_waves) return;
    const int lane = threadIdx.x % kWave;
    const int sub = lane % G;
    const uint32_t list_pos = id / kWavesPerChunk;
    const int64_t chunk = stream_chunks ? stream_chunks[list_pos] : (int64_t)list_pos;
    const int64_t row = chunk * kStreamRows + (id % kWavesPerChunk) * kRowsPerWave + lane / G;
    const bool row_ok = row < nrows;
    const int64_t row_c = row_ok ? row : nrows - 1;
    const int32_t p0 = rowptr[row_c], p1 = rowptr[row_c + 1];
    int32_t pat_begin = 0, pat_len = 0, pat_start = 0, pat_shift = 0;
    if constexpr (kHasPatterns) {
        pat_begin = pats.pat_off[chunk];
        pat_len = pats.pat_off[chunk + 1] - pat_begin;                  // wave-uniform
        const int32_t packed = pats.row_pat[row_c];
        pat_start = pattern_start(packed);
        pat_shift = pattern_shift(packed);
    }
    const bool patterned = RAW == kColsPattern || (RAW == kColsPatternOr16 && pat_len > 0);
    int32_t cbase = -1;                                                 // wave-uniform
    if constexpr (RAW != kColsPattern) {
        cbase = chunk_base ? chunk_base[chunk] : -1;
        if constexpr (RAW != kColsNarrow) {
            if (!patterned) load_frame_table(frame_table, chunk, cbase, lane, s_tab);
        }
    }
    if (patterned) {
        // the table is written once and read by every window of this wavefront's rows; all of
        // its loads are issued before the first is stored
        constexpr int kLoads = kPatternTable / kWave;
        int32_t d[kLoads];
#pragma unroll
        for (int i = 0; i < kLoads; ++i)
            if (i == 0 || i * kWave < pat_len) d[i] = (i * kWave + lane < pat_len) ? pats.pool[pat_begin + i * kWave + lane] : 0;
#pragma unroll
        for (int i = 0; i < kLoads; ++i)
            if (i == 0 || i * kWave < pat_len) s_pat[i * kWave + lane] = d[i];
    }
    const int32_t rb = row_ok ? p0 : p1, re = p1;      // rows past the end: empty range
    const int32_t base = __builtin_amdgcn_readfirstlane(rb);
    const int32_t end = __builtin_amdgcn_readlane(re, kWave - 1);
    const int32_t nnz4 = nnz & ~3;

    T s = T(0);
    // windows of kStreamWindow entries starting at a multiple of 8 (16-byte aligned loads of values,
    // 32-bit columns and 16-bit offsets alike)
    for (int32_t w0 = base & ~7; w0 < end; w0 += kStreamWindow) {      // uniform; one trip unless
        const int32_t w1 = (end - w0 < kStreamWindow) ? end : w0 + kStreamWindow;  // rows are dense
        if (patterned) stream_values_to_lds<T>(vals, w0, w1, nnz4, lane, s_val);
        else stream_window_to_lds<T, idx_t>(colidx, col16, cbase, s_tab, vals, w0, w1, nnz4, lane, s_col, s_val);

        // this lane's share of its row inside the window: entries ub+sub, ub+sub+G, ...
        const int32_t ub = (rb > w0 ? rb : w0) - w0;
        const int32_t ue = (re < w1 ? re : w1) - w0;
        const int my_n = (ue - ub - sub + G - 1) / G;                  // <= 0: nothing to do
        // Idle lanes re-read the first entry of the window that belongs to this wavefront's rows.
        // Not entry 0: the window starts at a multiple of 8, so its first entries may belong to the
        // previous chunk, whose 16-bit code decoded with this chunk's base or frame table can name a
        // column past the end of x.
        const int32_t own0 = (base > w0 ? base : w0) - w0;             // uniform
        const int first = my_n > 0 ? ub + sub : own0;
        if (patterned) {
            // the diagonals of the row's pattern from where this window cuts into the row; idle
            // lanes read the table's first diagonal and gather x[0]
            const int32_t *sc = s_pat + (my_n > 0 ? pat_start + (ub + w0 - rb) + sub : 0);
            const T *xb = my_n > 0 ? x + (row_c + pat_shift) : x - s_pat[0];
            s = stream_share<T, G, int32_t, kCols32, UNR>(sc, s_val + first, my_n, xb, nullptr, 0, s);
        } else {
            const T *xb = RAW == kColsNarrow ? x + cbase : x;
            s = stream_share<T, G, idx_t, kShareMode, UNR>(s_col + first, s_val + first, my_n, xb, s_tab, cbase, s);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    s = group_sum<G>(s);
    if (sub == G - 1 && row_ok) store_result(y, (int32_t)row, s, alpha, beta);
}

// ---- the paper's own kernel shape --------------------------------------------
// What the loop mapping of Section 4.2 produces for the CSR loop nest on a 64-lane
// back end: every row gets the same vector length G (one value per matrix, the
// average row length rounded up, clamped to the wavefront and, here, rounded up
// to a power of two), the ThreadVector lanes stride the row ("Loop translation",
// depth 2), the lane sums are reduced and one lane stores y[i] (`single`).  No
// row partition is used.  Kept beside the tuned kernels as the reference point.
template <typename T, int G>
__global__ __launch_bounds__(kBlock) void spmv_vector_kernel(
    int32_t nrows, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx,
    const T *__restrict__ vals, const T *__restrict__ x, T *__restrict__ y, T alpha, T beta)
{
    constexpr int kGroups = kBlock / G;
    const int lane = threadIdx.x % G;
    const int64_t row = (int64_t)blockIdx.x * kGroups + threadIdx.x / G;
    T s = T(0);
    if (row < nrows) {
        const int64_t je = rowptr[row + 1];
        for (int64_t j = (int64_t)rowptr[row] + lane; j < je; j += G) s += vals[j] * x[colidx[j]];
    }
    s = group_sum<G>(s);
    if (lane == G - 1 && row < nrows) store_result(y, (int32_t)row, s, alpha, beta);
}

// ---- long rows -------------------------------------------------------------
// Tile t covers positions [t*TILE, (t+1)*TILE) of the long rows' entries laid
// end to end.  Since every long row has more than TILE entries, a tile touches
// the row it starts in (segment A) and at most the next one (segment B).
// partial[2t] / partial[2t+1] receive the two segment sums.
template <typename T, int TILE>
__global__ __launch_bounds__(kBlock) void spmv_long_tile_kernel(
    int32_t num_long, const int32_t *__restrict__ long_rows, const int32_t *__restrict__ long_off,
    const int32_t *__restrict__ tile_row, const int32_t *__restrict__ tile_nz,
    const int32_t *__restrict__ row_begin, const int32_t *__restrict__ colidx,
    const T *__restrict__ vals, const T *__restrict__ x, T *__restrict__ partial)
{
    constexpr int kPerThread = TILE / kBlock;
    static_assert(TILE % kBlock == 0, "tile must be a multiple of the workgroup size");
    __shared__ T red[2 * kWavesPerBlock];

    const uint32_t t = blockIdx.x;
    const int32_t ra = tile_row[t];
    const int32_t za = tile_nz[t];
    const int64_t total = long_off[num_long];
    const int64_t tile_begin = (int64_t)t * TILE;
    const int64_t tile_len = (total - tile_begin < TILE) ? (total - tile_begin) : TILE;
    const int64_t len_a_row = long_off[ra + 1] - long_off[ra];
    const int64_t len_a = (len_a_row - za < tile_len) ? (len_a_row - za) : tile_len;
    const int64_t ja = (int64_t)row_begin[long_rows[ra]] + za;        // first entry of segment A
    const int64_t jb = (len_a < tile_len) ? (int64_t)row_begin[long_rows[ra + 1]] : 0;  // segment B

    int32_t c[kPerThread];
    T v[kPerThread];
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
        const int64_t p = (int64_t)i * kBlock + threadIdx.x;
        const int64_t j = (p < len_a) ? ja + p : jb + (p - len_a);
        const bool in = p < tile_len;
        c[i] = in ? load_stream(colidx + j) : -1;
        v[i] = in ? load_stream(vals + j) : T(0);
    }
    T sa = T(0), sb = T(0);
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
        const int64_t p = (int64_t)i * kBlock + threadIdx.x;
        const T prod = (c[i] >= 0) ? v[i] * x[c[i]] : T(0);
        if (p < len_a) sa += prod; else sb += prod;
    }
    sa = group_sum<kWave>(sa);
    sb = group_sum<kWave>(sb);
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    if (lane == kWave - 1) { red[2 * wave] = sa; red[2 * wave + 1] = sb; }
    __syncthreads();
    if (threadIdx.x < 2) {
        T s = T(0);
#pragma unroll
        for (int w = 0; w < kWavesPerBlock; ++w) s += red[2 * w + threadIdx.x];
        partial[2 * (int64_t)t + threadIdx.x] = s;
    }
}

// One wavefront per long row: add the row's tile sums (lanes stride the tiles
// in a fixed pattern, then a fixed reduction tree) and write y once.
template <typename T, int TILE>
__global__ __launch_bounds__(kBlock) void spmv_long_fixup_kernel(
    int32_t num_long, const int32_t *__restrict__ long_rows, const int32_t *__restrict__ long_off,
    const int32_t *__restrict__ tile_row, const T *__restrict__ partial, T *__restrict__ y,
    T alpha, T beta)
{
    const int64_t r = (int64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
    const int lane = threadIdx.x % kWave;
    T s = T(0);
    if (r < num_long) {
        const int64_t first = long_off[r] / TILE;
        const int64_t last = ((int64_t)long_off[r + 1] - 1) / TILE;
        for (int64_t t = first + lane; t <= last; t += kWave)
            s += partial[2 * t + (tile_row[t] == r ? 0 : 1)];
    }
    s = group_sum<kWave>(s);
    if (lane == kWave - 1 && r < num_long) store_result(y, long_rows[r], s, alpha, beta);
}

// ---- huge rows: column blocks of x staged in LDS ---------------------------------
// Rows above LAPIS_HUGE_ROW entries with ascending columns are cut at the boundaries of column
// blocks that hold LAPIS_LDS_BLOCK_BYTES of x (fcut, H rows x (nbf + 1) cuts).  Workgroup
// (b, g) copies block b of x into LDS once and then walks the pieces of its share of the rows:
// a piece is a contiguous run of colidx / vals, read with coalesced loads, and its gathers of x
// are LDS reads instead of one cache line per entry.  fsum[b*H + h] receives the piece's sum.
constexpr int kLdsBlockThreads = 1024;
constexpr int kLdsBlockWaves = kLdsBlockThreads / kWave;
constexpr int kLdsBlockUnroll = 4;            // loads of 64 entries in flight per wavefront

template <typename T>
__global__ __launch_bounds__(kLdsBlockThreads) void spmv_ldsblock_kernel(
    int32_t H, int32_t fblock_width, int64_t ncols, const int32_t *__restrict__ fcut,
    const int32_t *__restrict__ colidx, const T *__restrict__ vals, const T *__restrict__ x,
    T *__restrict__ fsum)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char s_raw[];
    T *s_x = reinterpret_cast<T *>(s_raw);
    const int32_t b = blockIdx.x;
    const int64_t c0 = (int64_t)b * fblock_width;
    const int32_t width = (int32_t)((ncols - c0 < fblock_width) ? ncols - c0 : fblock_width);
    for (int32_t i = threadIdx.x; i < width; i += kLdsBlockThreads) s_x[i] = x[c0 + i];
    __syncthreads();
    const int lane = threadIdx.x % kWave;
    const int32_t stride = kLdsBlockWaves * (int32_t)gridDim.y;
    const int32_t *__restrict__ cut_lo = fcut + (int64_t)b * H;
    const int32_t *__restrict__ cut_hi = cut_lo + H;
    int32_t h = (int32_t)blockIdx.y * kLdsBlockWaves + (int32_t)(threadIdx.x / kWave);
    int32_t jb = 0, je = 0;
    if (h < H) { jb = cut_lo[h]; je = cut_hi[h]; }
    while (h < H) {                                    // uniform per wavefront
        const int32_t h_next = h + stride;
        int32_t jb_next = 0, je_next = 0;
        if (h_next < H) { jb_next = cut_lo[h_next]; je_next = cut_hi[h_next]; }   // on its way during the piece
        T s = T(0);
        for (int32_t j0 = jb; j0 < je; j0 += kLdsBlockUnroll * kWave) {
            int32_t c[kLdsBlockUnroll];
            T v[kLdsBlockUnroll];
#pragma unroll
            for (int q = 0; q < kLdsBlockUnroll; ++q) {
                const int32_t j = j0 + q * kWave + lane;
                const int32_t jc = j < je ? j : je - 1;                 // past the end: the last entry again
                c[q] = load_stream(colidx + jc);
                v[q] = load_stream(vals + jc);
            }
#pragma unroll
            for (int q = 0; q < kLdsBlockUnroll; ++q) {
                const T p = v[q] * s_x[c[q] - (int32_t)c0];
                s += (j0 + q * kWave + lane < je) ? p : T(0);
            }
        }
        s = group_sum<kWave>(s);
        if (lane == kWave - 1) fsum[(int64_t)b * H + h] = s;
        h = h_next; jb = jb_next; je = je_next;
    }
}

// One wavefront per huge row: y[row] = alpha * (sum over the blocks of fsum[b*H + h]) + beta * y[row];
// lanes stride the blocks in a fixed pattern, then a fixed reduction tree.
template <typename T>
__global__ __launch_bounds__(kBlock) void spmv_ldsblock_combine_kernel(
    int32_t H, int32_t nbf, const int32_t *__restrict__ huge_rows, const T *__restrict__ fsum,
    T *__restrict__ y, T alpha, T beta)
{
    const int64_t h = (int64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
    const int lane = threadIdx.x % kWave;
    T s = T(0);
    if (h < H)
        for (int32_t b = lane; b < nbf; b += kWave) s += fsum[(int64_t)b * H + h];
    s = group_sum<kWave>(s);
    if (lane == kWave - 1 && h < H) store_result(y, huge_rows[h], s, alpha, beta);
}

}  // namespace lapis
