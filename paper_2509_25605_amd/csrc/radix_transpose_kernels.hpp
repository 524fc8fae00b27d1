// Explicit transposition (the CSR arrays of A^T on the device) by a stable radix sort of the
// entries by column: the entries of one column then appear in the order of their entry ids,
// which is the order a serial row-by-row transposition produces (duplicates included), with no
// atomics in memory and no order left to chance.
//   keys = colidx, values = entry ids -> one pass per 8 bits of the largest column, lowest bits
//   first: per-wavefront digit counts -> exclusive scan over (digit, wavefront) -> every
//   wavefront moves its entries to their places, keeping their order -> tptr from the sorted
//   columns -> rows and values of the entries gathered through the sorted ids.
#pragma once
#include "analysis_kernels.hpp"

namespace lapis {

constexpr int kRadixBits = 8;
constexpr int kRadixDigits = 1 << kRadixBits;
constexpr int kRadixPerWave = 8192;                  // consecutive entries one wavefront owns
constexpr int kRadixGroup = 16;                      // steps of 64 entries whose loads are issued together
constexpr int kRadixTile = kRadixPerWave * kWavesPerBlock;

// count[digit * num_waves + w] = how many of the entries of wavefront w (entries
// w * kRadixPerWave ...) have that digit; num_waves = ceil(n / kRadixPerWave).
__global__ __launch_bounds__(kBlock) void radix_count_kernel(int32_t n, int32_t num_waves, int shift,
                                                             const int32_t *__restrict__ keys,
                                                             int32_t *__restrict__ count)
{
    __shared__ int32_t s_count[kWavesPerBlock][kRadixDigits];
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    for (int d = lane; d < kRadixDigits; d += kWave) s_count[wave][d] = 0;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const int64_t w = (int64_t)blockIdx.x * kWavesPerBlock + wave;
    if (w >= num_waves) return;                        // whole wavefronts leave together
    const int64_t begin = w * kRadixPerWave;
    const int64_t end = begin + kRadixPerWave < n ? begin + kRadixPerWave : n;
    const uint64_t below = (1ull << lane) - 1;
    for (int64_t g0 = begin; g0 < end; g0 += kRadixGroup * kWave) {  // uniform
        int32_t k[kRadixGroup];
#pragma unroll
        for (int q = 0; q < kRadixGroup; ++q) {
            const int64_t j = g0 + q * kWave + lane;
            k[q] = j < end ? load_stream(keys + j) : 0;
        }
#pragma unroll
        for (int q = 0; q < kRadixGroup; ++q) {
            const bool valid = g0 + q * kWave + lane < end;
            const int d = (k[q] >> shift) & (kRadixDigits - 1);
            // sorted input puts many lanes on one digit: the first of them adds for all
            uint64_t same = __ballot(valid);
#pragma unroll
            for (int b = 0; b < kRadixBits; ++b) {
                const uint64_t has = __ballot((d >> b) & 1);
                same &= ((d >> b) & 1) ? has : ~has;
            }
            if (valid && (same & below) == 0) atomicAdd(&s_count[wave][d], (int32_t)__popcll(same));
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    for (int d = lane; d < kRadixDigits; d += kWave) count[(int64_t)d * num_waves + w] = s_count[wave][d];
}

// offset = exclusive scan of count (same indexing).  Every wavefront moves its entries, in their
// order, to offset[digit][w] + (how many of its earlier entries have the same digit).
// vals_in == nullptr: the value of entry j is j.
__global__ __launch_bounds__(kBlock) void radix_scatter_kernel(int32_t n, int32_t num_waves, int shift,
                                                               const int32_t *__restrict__ keys_in,
                                                               const int32_t *__restrict__ vals_in,
                                                               const int32_t *__restrict__ offset,
                                                               int32_t *__restrict__ keys_out,
                                                               int32_t *__restrict__ vals_out)
{
    __shared__ int32_t s_base[kWavesPerBlock][kRadixDigits];
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int64_t w = (int64_t)blockIdx.x * kWavesPerBlock + wave;
    if (w >= num_waves) return;                        // whole wavefronts leave together
    for (int d = lane; d < kRadixDigits; d += kWave) s_base[wave][d] = offset[(int64_t)d * num_waves + w];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const int64_t begin = w * kRadixPerWave;
    const int64_t end = begin + kRadixPerWave < n ? begin + kRadixPerWave : n;
    const uint64_t below = (1ull << lane) - 1;
    for (int64_t g0 = begin; g0 < end; g0 += kRadixGroup * kWave) {  // uniform
        // the loads of a group of steps are issued together, the steps then run from registers
        int32_t keys[kRadixGroup], vals[kRadixGroup];
#pragma unroll
        for (int q = 0; q < kRadixGroup; ++q) {
            const int64_t j = g0 + q * kWave + lane;
            keys[q] = j < end ? load_stream(keys_in + j) : 0;
            vals[q] = j < end ? (vals_in ? load_stream(vals_in + j) : (int32_t)j) : 0;
        }
#pragma unroll
        for (int q = 0; q < kRadixGroup; ++q) {
            const bool valid = g0 + q * kWave + lane < end;
            const int d = (keys[q] >> shift) & (kRadixDigits - 1);
            // the lanes with my digit
            uint64_t same = __ballot(valid);
#pragma unroll
            for (int b = 0; b < kRadixBits; ++b) {
                const uint64_t has = __ballot((d >> b) & 1);
                same &= ((d >> b) & 1) ? has : ~has;
            }
            const int32_t base = s_base[wave][d];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const int rank = __popcll(same & below);
            if (valid) {
                if (rank == 0) s_base[wave][d] = base + __popcll(same);     // one lane per digit
                keys_out[base + rank] = keys[q];
                vals_out[base + rank] = vals[q];
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
    }
}

// tptr[c] = first position of the sorted entries whose column is >= c, c = 0 .. ncols.
__global__ __launch_bounds__(kBlock) void sorted_keys_to_ptr_kernel(int32_t n, int32_t ncols,
                                                                    const int32_t *__restrict__ sorted_keys,
                                                                    int32_t *__restrict__ tptr)
{
    for (int64_t p = (int64_t)blockIdx.x * kBlock + threadIdx.x; p <= n; p += (int64_t)gridDim.x * kBlock) {
        const int32_t prev = p > 0 ? sorted_keys[p - 1] : -1;
        const int32_t cur = p < n ? sorted_keys[p] : ncols;
        for (int32_t c = prev + 1; c <= cur; ++c) tptr[c] = (int32_t)p;
    }
}

// row[j] = the row that holds entry j, for a tile of kCheckTile entries per workgroup (the rows
// that start inside the tile leave their id at their first entry's slot in LDS, a running
// maximum spreads it).  tile_first comes from check_tile_rows_kernel.
__global__ __launch_bounds__(kBlock) void entry_rows_kernel(int32_t nnz, const int32_t *__restrict__ rowptr,
                                                            const int32_t *__restrict__ tile_first,
                                                            int32_t *__restrict__ row)
{
    constexpr int kPer = kCheckTile / kBlock;
    __shared__ int32_t s_row[kCheckTile];
    __shared__ int32_t s_scan[kBlock];
    const int tid = threadIdx.x;
    for (int64_t t = blockIdx.x; t * kCheckTile < nnz; t += gridDim.x) {
        const int32_t j0 = (int32_t)(t * kCheckTile);
        const int32_t j1 = (int32_t)((t * kCheckTile + kCheckTile < nnz) ? t * kCheckTile + kCheckTile : nnz);
        const int32_t first = tile_first[t], next = tile_first[t + 1];
        __syncthreads();
#pragma unroll
        for (int i = 0; i < kPer; ++i) s_row[i * kBlock + tid] = first;
        __syncthreads();
        for (int64_t r = (int64_t)first + 1 + tid; r <= next; r += kBlock) {
            const int32_t at = rowptr[r];
            if (at > j0 && at < j1) atomicMax(&s_row[at - j0], (int32_t)r);
        }
        __syncthreads();
        int32_t v[kPer];
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            v[i] = s_row[tid * kPer + i];
            if (i > 0) v[i] = max(v[i], v[i - 1]);
        }
        s_scan[tid] = v[kPer - 1];
        __syncthreads();
        for (int d = 1; d < kBlock; d *= 2) {
            const int32_t other = tid >= d ? s_scan[tid - d] : 0;
            __syncthreads();
            s_scan[tid] = max(s_scan[tid], other);
            __syncthreads();
        }
        const int32_t before = tid > 0 ? s_scan[tid - 1] : 0;
#pragma unroll
        for (int i = 0; i < kPer; ++i) s_row[tid * kPer + i] = max(v[i], before);
        __syncthreads();
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const int32_t pos = i * kBlock + tid;
            if (j0 + pos < j1) row[j0 + pos] = s_row[pos];
        }
    }
}

// tidx[p] = row of the entry that lands at position p, tvals[p] = its value
template <typename T>
__global__ __launch_bounds__(kBlock) void transpose_gather_sorted_kernel(int32_t nnz, const int32_t *__restrict__ entry,
                                                                         const int32_t *__restrict__ entry_row,
                                                                         const T *__restrict__ vals,
                                                                         int32_t *__restrict__ tidx, T *__restrict__ tvals)
{
    for (int64_t p = (int64_t)blockIdx.x * kBlock + threadIdx.x; p < nnz; p += (int64_t)gridDim.x * kBlock) {
        const int32_t e = load_stream(entry + p);
        tidx[p] = entry_row[e];
        tvals[p] = vals[e];
    }
}

}  // namespace lapis
