// y = alpha * A^T x + beta * y from the CSR arrays of A: the column-wise (CSC) traversal of the
// sparse loop pattern of Section 4.2.  The CSR arrays of A are the CSC arrays of A^T, so entry j
// of row i adds vals[j] * x[i] into y[colidx[j]]: the matrix is streamed once with coalesced
// loads, in tiles of consecutive entries, and the sums are formed by hardware floating-point
// atomics in memory.  The order of the additions into one y element is not fixed, so results
// agree with a serial evaluation only up to the rounding bound, and may differ between runs.
#pragma once
#include "analysis_kernels.hpp"

namespace lapis {

constexpr int kScatterPerThread = 8;
constexpr int kScatterTile = kBlock * kScatterPerThread;     // entries per workgroup
constexpr int kScatterRowsInLds = kScatterTile + 2;          // row starts of a tile without empty rows

// y = beta * y (exactly 0 when beta == 0, whatever y held)
template <typename T>
__global__ __launch_bounds__(kBlock) void transpose_scale_kernel(int64_t n, T *__restrict__ y, T b)
{
    for (int64_t c = (int64_t)blockIdx.x * kBlock + threadIdx.x; c < n; c += (int64_t)gridDim.x * kBlock)
        y[c] = (b == T(0)) ? T(0) : b * y[c];
}

// Rows touched by a workgroup's tile of consecutive entries [j0, j1): [first, last]; their starts
// are staged in LDS when they fit (no long run of empty rows inside), so that each entry finds its
// row by bisection there instead of in memory.
struct TileRows {
    int32_t first, last;
    bool staged;
};

// largest r in [lo, hi] with start(r) <= j; rows before it that start at the same entry are empty
template <typename F>
__device__ __forceinline__ int32_t last_row_starting_at_or_before(F start, int32_t j, int32_t lo, int32_t hi)
{
    while (lo < hi) {
        const int32_t mid = lo + (hi - lo + 1) / 2;
        if (start(mid) <= j) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// Whole workgroup; s_start has kScatterRowsInLds ints, s_range 2.  nrows >= 1, j0 < j1 <= nnz.
__device__ __forceinline__ TileRows stage_tile_rows(int32_t *s_start, int32_t *s_range, int32_t j0, int32_t j1,
                                                    int32_t nrows, const int32_t *__restrict__ rowptr)
{
    auto global_start = [&](int32_t r) { return rowptr[r]; };
    if (threadIdx.x < 2)
        s_range[threadIdx.x] =
            last_row_starting_at_or_before(global_start, threadIdx.x == 0 ? j0 : j1 - 1, 0, nrows - 1);
    __syncthreads();
    TileRows t;
    t.first = s_range[0];
    t.last = s_range[1];
    t.staged = t.last - t.first + 1 <= kScatterRowsInLds;
    if (t.staged)
        for (int32_t r = t.first + (int32_t)threadIdx.x; r <= t.last; r += kBlock) s_start[r - t.first] = rowptr[r];
    __syncthreads();
    return t;
}

__device__ __forceinline__ int32_t tile_row_of(const TileRows &t, const int32_t *s_start,
                                               const int32_t *__restrict__ rowptr, int32_t j)
{
    if (t.staged)
        return last_row_starting_at_or_before([&](int32_t r) { return s_start[r - t.first]; }, j, t.first, t.last);
    return last_row_starting_at_or_before([&](int32_t r) { return rowptr[r]; }, j, t.first, t.last);
}

// One workgroup per tile of kScatterTile consecutive entries.
// nrows >= 1, nnz >= 1, rowptr valid (checked when the handle was created).
template <typename T>
__global__ __launch_bounds__(kBlock) void transpose_scatter_kernel(int32_t nrows, int32_t nnz,
                                                                   const int32_t *__restrict__ rowptr,
                                                                   const int32_t *__restrict__ colidx,
                                                                   const T *__restrict__ vals,
                                                                   const T *__restrict__ x, T *__restrict__ y, T a)
{
    __shared__ int32_t s_start[kScatterRowsInLds];
    __shared__ int32_t s_range[2];
    const int32_t j0 = (int32_t)blockIdx.x * kScatterTile;
    const int32_t j1 = (nnz - j0 > kScatterTile) ? j0 + kScatterTile : nnz;
    const TileRows rows = stage_tile_rows(s_start, s_range, j0, j1, nrows, rowptr);

    int32_t c[kScatterPerThread];
    T v[kScatterPerThread];
#pragma unroll
    for (int k = 0; k < kScatterPerThread; ++k) {
        const int32_t j = j0 + k * kBlock + (int32_t)threadIdx.x;
        const int32_t jc = j < j1 ? j : j1 - 1;           // clamped: always a valid entry
        c[k] = load_stream(colidx + jc);
        v[k] = load_stream(vals + jc);
    }
#pragma unroll
    for (int k = 0; k < kScatterPerThread; ++k) {
        const int32_t j = j0 + k * kBlock + (int32_t)threadIdx.x;
        if (j < j1) unsafeAtomicAdd(y + c[k], a * (v[k] * x[tile_row_of(rows, s_start, rowptr, j)]));
    }
}

// ---- explicit transposition: the CSR arrays of A^T, built on the device ------
// count the entries of every column -> exclusive scan gives tptr -> every entry takes a slot of
// its column with an atomic cursor (any order) and leaves the key (column, entry id) and its row
// -> the slots of each column are sorted by entry id, which is the order of a serial row-by-row
// transposition (unique, duplicates included) -> values are gathered through the entry ids.
// Columns of at most kSortHalf entries are sorted in LDS, several columns per workgroup; longer
// ones by one workgroup each in memory.

// count[c] = entries in column c; count must be 0 on entry
__global__ __launch_bounds__(kBlock) void column_count_kernel(int32_t nnz, const int32_t *__restrict__ colidx,
                                                              int32_t *__restrict__ count)
{
    for (int64_t j = (int64_t)blockIdx.x * kBlock + threadIdx.x; j < nnz; j += (int64_t)gridDim.x * kBlock)
        atomicAdd(&count[load_stream(colidx + j)], 1);
}

// Exclusive scan of n ints in three launches: per-tile sums, scan of the sums by one workgroup,
// per-tile scan with the tile's offset.  out has n + 1 elements (out[n] = total).
constexpr int kScanPerThread = 8;
constexpr int kScanTile = kBlock * kScanPerThread;

// sum over the wavefront, in lane 63
__device__ __forceinline__ int32_t wave_sum_int(int32_t v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x141, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x140, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);
    return v;
}

__global__ __launch_bounds__(kBlock) void scan_tile_sums_kernel(int64_t n, const int32_t *__restrict__ in,
                                                                int32_t *__restrict__ tile_sum)
{
    __shared__ int32_t s_tmp[kWavesPerBlock];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanPerThread;
    int32_t v = 0;
#pragma unroll
    for (int q = 0; q < kScanPerThread; ++q) v += (base + q < n) ? in[base + q] : 0;
    v = wave_sum_int(v);
    if (threadIdx.x % kWave == kWave - 1) s_tmp[threadIdx.x / kWave] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        int32_t total = 0;
        for (int w = 0; w < kWavesPerBlock; ++w) total += s_tmp[w];
        tile_sum[blockIdx.x] = total;
    }
}

// one workgroup: tile_sum[0..num_tiles) -> exclusive prefix in place, tile_sum[num_tiles] = total
__global__ __launch_bounds__(kBlock) void scan_tile_offsets_kernel(int32_t num_tiles, int32_t *__restrict__ tile_sum)
{
    __shared__ int32_t s_tmp[kBlock];
    int32_t running = 0;
    for (int64_t base = 0; base < num_tiles; base += kBlock) {
        const int64_t i = base + threadIdx.x;
        const int32_t v = (i < num_tiles) ? tile_sum[i] : 0;
        int32_t total;
        const int32_t excl = block_exclusive_scan(v, s_tmp, &total);
        if (i < num_tiles) tile_sum[i] = running + excl;
        running += total;
    }
    if (threadIdx.x == 0) tile_sum[num_tiles] = running;
}

__global__ __launch_bounds__(kBlock) void scan_apply_kernel(int64_t n, const int32_t *__restrict__ in,
                                                            const int32_t *__restrict__ tile_offset,
                                                            int32_t num_tiles, int32_t *__restrict__ out)
{
    __shared__ int32_t s_tmp[kBlock];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanPerThread;
    int32_t v[kScanPerThread];
    int32_t mine = 0;
#pragma unroll
    for (int q = 0; q < kScanPerThread; ++q) {
        v[q] = (base + q < n) ? in[base + q] : 0;
        mine += v[q];
    }
    int32_t total;
    int32_t prefix = tile_offset[blockIdx.x] + block_exclusive_scan(mine, s_tmp, &total);
#pragma unroll
    for (int q = 0; q < kScanPerThread; ++q) {
        if (base + q < n) out[base + q] = prefix;
        prefix += v[q];
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) out[n] = tile_offset[num_tiles];
}

// Every entry j (row r, column c) takes slot p = tptr[c] + (cursor[c]++) and leaves
// key[p] = (c << 32) | j and trow[p] = r.  cursor must be 0 on entry.  Same tiling as the scatter.
__global__ __launch_bounds__(kBlock) void transpose_fill_kernel(int32_t nrows, int32_t nnz,
                                                                const int32_t *__restrict__ rowptr,
                                                                const int32_t *__restrict__ colidx,
                                                                const int32_t *__restrict__ tptr,
                                                                int32_t *__restrict__ cursor,
                                                                uint64_t *__restrict__ key, int32_t *__restrict__ trow)
{
    __shared__ int32_t s_start[kScatterRowsInLds];
    __shared__ int32_t s_range[2];
    const int32_t j0 = (int32_t)blockIdx.x * kScatterTile;
    const int32_t j1 = (nnz - j0 > kScatterTile) ? j0 + kScatterTile : nnz;
    const TileRows rows = stage_tile_rows(s_start, s_range, j0, j1, nrows, rowptr);
#pragma unroll
    for (int k = 0; k < kScatterPerThread; ++k) {
        const int32_t j = j0 + k * kBlock + (int32_t)threadIdx.x;
        if (j < j1) {
            const int32_t c = load_stream(colidx + j);
            const int32_t p = tptr[c] + atomicAdd(&cursor[c], 1);
            key[p] = ((uint64_t)(uint32_t)c << 32) | (uint32_t)j;
            trow[p] = tile_row_of(rows, s_start, rowptr, j);
        }
    }
}

constexpr int kSortHalf = 1024;             // longest column sorted in LDS; also the slot range per workgroup
constexpr int kSortTile = 2 * kSortHalf;    // most slots one workgroup can meet
constexpr uint64_t kSortPad = ~0ull;

// first column c in [0, ncols] with tptr[c] >= p   (tptr[ncols] = nnz >= p)
__device__ __forceinline__ int32_t first_column_starting_at_or_after(const int32_t *__restrict__ tptr,
                                                                     int32_t ncols, int32_t p)
{
    int32_t lo = 0, hi = ncols;
    while (lo < hi) {
        const int32_t mid = lo + (hi - lo) / 2;
        if (tptr[mid] >= p) hi = mid; else lo = mid + 1;
    }
    return lo;
}

// The comparators of a sorting network on indices [0, np), np a power of two, that orders every
// pair ascending (merge steps start with a mirrored partner), so positions padded with the
// largest key never move.  step(i, partner) is called for i < partner; `sync` between levels.
template <typename Step, typename Sync>
__device__ __forceinline__ void ascending_network(int32_t np, int32_t threads, Step step, Sync sync)
{
    for (int32_t k = 2; k <= np; k <<= 1) {
        for (int32_t t = threadIdx.x; t < np / 2; t += threads) {
            const int32_t half = k >> 1, blk = t / half, off = t % half;
            step(blk * k + off, blk * k + k - 1 - off);
        }
        sync();
        for (int32_t d = k >> 2; d > 0; d >>= 1) {
            for (int32_t t = threadIdx.x; t < np / 2; t += threads) {
                const int32_t i = 2 * d * (t / d) + t % d;
                step(i, i + d);
            }
            sync();
        }
    }
}

// Workgroup t owns the columns whose first slot lies in [t*kSortHalf, (t+1)*kSortHalf).  Only the
// last of them can be longer than kSortHalf; it is then left out and appended to long_cols (in
// any order).  The rest, fewer than kSortTile slots, is sorted by key in LDS: the column is the
// major part of the key, so every column ends up sorted by entry id in its own slots.
__global__ __launch_bounds__(kBlock) void transpose_sort_tiles_kernel(int32_t ncols, int32_t nnz,
                                                                      const int32_t *__restrict__ tptr,
                                                                      uint64_t *__restrict__ key,
                                                                      int32_t *__restrict__ trow,
                                                                      int32_t *__restrict__ long_cols,
                                                                      int32_t *__restrict__ num_long)
{
    __shared__ uint64_t s_key[kSortTile];
    __shared__ int32_t s_row[kSortTile];
    __shared__ int32_t s_col[2];
    const int32_t lo = (int32_t)blockIdx.x * kSortHalf;
    const int32_t hi = (nnz - lo > kSortHalf) ? lo + kSortHalf : nnz;
    if (threadIdx.x < 2) s_col[threadIdx.x] = first_column_starting_at_or_after(tptr, ncols, threadIdx.x == 0 ? lo : hi);
    __syncthreads();
    const int32_t c_first = s_col[0], c_end = s_col[1];
    if (c_first >= c_end) return;                       // no column starts here (inside a long column)
    const int32_t c_last = c_end - 1;
    const int32_t last_begin = tptr[c_last], last_end = tptr[c_last + 1];
    const bool last_is_long = last_end - last_begin > kSortHalf;
    if (last_is_long && threadIdx.x == 0) long_cols[atomicAdd(num_long, 1)] = c_last;
    const int32_t p0 = tptr[c_first];
    const int32_t n = (last_is_long ? last_begin : last_end) - p0;     // < kSortTile
    if (n <= 1) return;
    int32_t np = 2;
    while (np < n) np <<= 1;
    for (int32_t i = threadIdx.x; i < np; i += kBlock) {
        s_key[i] = (i < n) ? key[p0 + i] : kSortPad;
        s_row[i] = (i < n) ? trow[p0 + i] : 0;
    }
    __syncthreads();
    ascending_network(
        np, kBlock,
        [&](int32_t i, int32_t partner) {
            const uint64_t a = s_key[i], b = s_key[partner];
            if (a > b) {
                s_key[i] = b; s_key[partner] = a;
                const int32_t ra = s_row[i];
                s_row[i] = s_row[partner]; s_row[partner] = ra;
            }
        },
        [] { __syncthreads(); });
    for (int32_t i = threadIdx.x; i < n; i += kBlock) {
        key[p0 + i] = s_key[i];
        trow[p0 + i] = s_row[i];
    }
}

// One workgroup of kSortLongBlock threads per column longer than kSortHalf: the same network on the
// column's slots in memory (comparators that reach beyond the column's end meet the padding and
// are skipped).
constexpr int kSortLongBlock = 1024;
__global__ __launch_bounds__(kSortLongBlock) void transpose_sort_long_kernel(const int32_t *__restrict__ long_cols,
                                                                             const int32_t *__restrict__ tptr,
                                                                             uint64_t *key, int32_t *trow)
{
    const int32_t c = long_cols[blockIdx.x];
    const int32_t p0 = tptr[c], n = tptr[c + 1] - p0;
    int32_t np = 2;
    while (np < n) np <<= 1;
    uint64_t *k = key + p0;
    int32_t *r = trow + p0;
    ascending_network(
        np, kSortLongBlock,
        [&](int32_t i, int32_t partner) {
            if (partner < n) {
                const uint64_t a = k[i], b = k[partner];
                if (a > b) {
                    k[i] = b; k[partner] = a;
                    const int32_t ra = r[i];
                    r[i] = r[partner]; r[partner] = ra;
                }
            }
        },
        [] { __syncthreads(); });
}

// tvals[p] = vals[entry id of slot p]
template <typename T>
__global__ __launch_bounds__(kBlock) void transpose_gather_kernel(int32_t nnz, const uint64_t *__restrict__ key,
                                                                  const T *__restrict__ vals, T *__restrict__ tvals)
{
    for (int64_t p = (int64_t)blockIdx.x * kBlock + threadIdx.x; p < nnz; p += (int64_t)gridDim.x * kBlock)
        tvals[p] = vals[(uint32_t)load_stream(key + p)];
}

}  // namespace lapis
