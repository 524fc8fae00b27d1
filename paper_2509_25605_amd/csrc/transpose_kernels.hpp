// y = alpha * A^T x + beta * y from the CSR arrays of A: the column-wise (CSC) traversal of the
// sparse loop pattern of Section 4.2.  The CSR arrays of A are the CSC arrays of A^T, so entry j
// of row i adds vals[j] * x[i] into y[colidx[j]]: the matrix is streamed once with coalesced
// loads, in tiles of consecutive entries, and the sums are formed by hardware floating-point
// atomics in memory.  The order of the additions into one y element is not fixed, so results
// agree with a serial evaluation only up to the rounding bound, and may differ between runs.
#pragma once
#include "device_utils.hpp"

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

// One workgroup per tile of kScatterTile consecutive entries.  The rows the tile touches are
// [first, last]; their starts are staged in LDS when they fit (no run of empty rows inside), so
// each entry finds its row by bisection there instead of in memory.
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
    // largest r in [lo, hi] with start(r) <= j; rows before it that start at the same entry are empty
    auto row_of = [](auto start, int32_t j, int32_t lo, int32_t hi) {
        while (lo < hi) {
            const int32_t mid = lo + (hi - lo + 1) / 2;
            if (start(mid) <= j) lo = mid; else hi = mid - 1;
        }
        return lo;
    };
    auto global_start = [&](int32_t r) { return rowptr[r]; };
    if (threadIdx.x < 2)
        s_range[threadIdx.x] = row_of(global_start, threadIdx.x == 0 ? j0 : j1 - 1, 0, nrows - 1);
    __syncthreads();
    const int32_t first = s_range[0], last = s_range[1];
    const bool staged = last - first + 1 <= kScatterRowsInLds;
    if (staged)
        for (int32_t r = first + (int32_t)threadIdx.x; r <= last; r += kBlock) s_start[r - first] = rowptr[r];
    __syncthreads();
    auto lds_start = [&](int32_t r) { return s_start[r - first]; };

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
        if (j < j1) {
            const int32_t r = staged ? row_of(lds_start, j, first, last) : row_of(global_start, j, first, last);
            unsafeAtomicAdd(y + c[k], a * (v[k] * x[r]));
        }
    }
}

}  // namespace lapis
