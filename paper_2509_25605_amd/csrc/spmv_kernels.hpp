// SpMV kernels for gfx950: y = alpha*A*x + beta*y with A in CSR (Section 6.2),
// rows walked with the CSR loop nest of Section 4.2.
//
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
#pragma once
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

struct ShortPlan {
    int32_t bin_begin[kShortBins];        // first position of bin b in row_perm
    int32_t bin_count[kShortBins];        // rows in bin b
    uint32_t block_begin[kShortBins + 1]; // logical workgroups of bin b: [block_begin[b], block_begin[b+1])
    uint32_t num_blocks;                  // block_begin[kShortBins]
    uint32_t padded_blocks;               // num_blocks rounded up to a multiple of the XCD count
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
                                           const int32_t *__restrict__ rowptr,
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
        jb[u] = (row[u] >= 0) ? rowptr[row[u]] : 0;
        je[u] = (row[u] >= 0) ? rowptr[row[u] + 1] : 0;
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
                                          const int32_t *__restrict__ rowptr,
                                          const int32_t *__restrict__ colidx,
                                          const T *__restrict__ vals, const T *__restrict__ x,
                                          T *__restrict__ y, T alpha, T beta)
{
    const int wave = threadIdx.x / kWave;
    const int lane = threadIdx.x % kWave;
    const int64_t idx = (int64_t)local_block * kWavesPerBlock + wave;
    const int32_t row = (idx < count) ? row_perm[begin + idx] : -1;
    const int64_t jb = (row >= 0) ? rowptr[row] : 0;
    const int64_t je = (row >= 0) ? rowptr[row + 1] : 0;
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

template <typename T, bool XCD_REMAP>
__global__ __launch_bounds__(kBlock) void spmv_short_kernel(
    ShortPlan plan, const int32_t *__restrict__ row_perm, const int32_t *__restrict__ rowptr,
    const int32_t *__restrict__ colidx, const T *__restrict__ vals, const T *__restrict__ x,
    T *__restrict__ y, T alpha, T beta)
{
    const uint32_t id = XCD_REMAP ? xcd_contiguous_id(blockIdx.x, plan.padded_blocks) : blockIdx.x;
    if (id >= plan.num_blocks) return;
    int bin = 0;
    while (id >= plan.block_begin[bin + 1]) ++bin;  // uniform over the workgroup
    const uint32_t local = id - plan.block_begin[bin];
    const int32_t begin = plan.bin_begin[bin], count = plan.bin_count[bin];
#define LAPIS_SHORT_CASE(B)                                                                     \
    case B:                                                                                     \
        short_rows<T, short_group_size(B), short_rows_per_group(B)>(local, begin, count,        \
            row_perm, rowptr, colidx, vals, x, y, alpha, beta);                                 \
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
        wave_rows<T>(local, begin, count, row_perm, rowptr, colidx, vals, x, y, alpha, beta);
        break;
    }
#undef LAPIS_SHORT_CASE
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
    const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx,
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
    const int64_t ja = (int64_t)rowptr[long_rows[ra]] + za;           // first entry of segment A
    const int64_t jb = (len_a < tile_len) ? (int64_t)rowptr[long_rows[ra + 1]] : 0;  // segment B

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

}  // namespace lapis
