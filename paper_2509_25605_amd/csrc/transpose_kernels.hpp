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

// ---- exclusive scan of ints (used by the radix sort of the explicit transposition) ------

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

}  // namespace lapis
