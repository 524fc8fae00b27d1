// Device-side helpers shared by the gfx950 kernels: lane-group reductions on
// the 64-lane wavefront and streaming loads.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lapis {

constexpr int kWave = 64;          // gfx950 wavefront width
constexpr int kBlock = 256;        // threads per workgroup used by every kernel here
constexpr int kWavesPerBlock = kBlock / kWave;

// One DPP move of a 32- or 64-bit value.  Lanes whose row is masked out by
// ROWMASK, and lanes whose source lane does not exist, receive 0.
template <int CTRL, int ROWMASK>
__device__ __forceinline__ float dpp_move(float v)
{
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROWMASK, 0xf, false));
}
template <int CTRL, int ROWMASK>
__device__ __forceinline__ double dpp_move(double v)
{
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __builtin_amdgcn_update_dpp(0, lo, CTRL, ROWMASK, 0xf, false);
    hi = __builtin_amdgcn_update_dpp(0, hi, CTRL, ROWMASK, 0xf, false);
    return __hiloint2double(hi, lo);
}

// Sum over aligned groups of G consecutive lanes (G a power of two <= 64).
// Every lane of the wavefront must be active.  The total is guaranteed in the
// LAST lane of each group (lane % G == G-1); for G <= 16 every lane holds it.
//   steps 1,2: quad permutes (lane ^ 1, lane ^ 2)
//   step 4:    row_half_mirror (lane -> 7 - lane within 8)
//   step 8:    row_mirror      (lane -> 15 - lane within 16)
//   step 16:   row_bcast:15 into rows 1 and 3
//   step 32:   row_bcast:31 into rows 2 and 3
template <int G, typename T>
__device__ __forceinline__ T group_sum(T v)
{
    static_assert(G >= 1 && G <= 64 && (G & (G - 1)) == 0, "group size must be a power of two");
    if constexpr (G >= 2) v += dpp_move<0xB1, 0xf>(v);
    if constexpr (G >= 4) v += dpp_move<0x4E, 0xf>(v);
    if constexpr (G >= 8) v += dpp_move<0x141, 0xf>(v);
    if constexpr (G >= 16) v += dpp_move<0x140, 0xf>(v);
    if constexpr (G >= 32) v += dpp_move<0x142, 0xa>(v);
    if constexpr (G >= 64) v += dpp_move<0x143, 0xc>(v);
    return v;
}

// Maximum of a non-negative int over the wavefront, returned as a wave-uniform value.
// Every lane must be active.
__device__ __forceinline__ int wave_max_nonneg(int v)
{
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xf, 0xf, false));
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xf, 0xf, false));
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x141, 0xf, 0xf, false));
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x140, 0xf, 0xf, false));
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false));   // rows 1, 3 <- lane 15 of rows 0, 2
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false));   // rows 2, 3 <- lane 31
    return __builtin_amdgcn_readlane(v, kWave - 1);
}

// Streaming load: data read once per product (values, column indices) is
// fetched with the non-temporal hint so it does not evict x from the caches.
template <typename T>
__device__ __forceinline__ T load_stream(const T *p)
{
    return __builtin_nontemporal_load(p);
}

// Workgroups are dealt round-robin to the 8 XCDs, each with a private L2.
// Map the hardware workgroup id to a logical id so that every XCD walks one
// contiguous range of logical ids (contiguous rows share x in that L2).
// `padded` is the grid size rounded up to a multiple of 8; ids >= the real
// count must be skipped by the caller.
constexpr int kXcds = 8;
__device__ __forceinline__ uint32_t xcd_contiguous_id(uint32_t hw_id, uint32_t padded)
{
    return (hw_id % kXcds) * (padded / kXcds) + hw_id / kXcds;
}

// Block-cyclic variant: logical ids are dealt to the XCDs in blocks of `block` consecutive ids
// (block b goes to XCD b % 8), and each XCD walks its blocks in ascending order.  With rows
// numbered along a band of half-width h and block = h/8 rows, the 8 XCDs share every band-wide
// window of rows instead of each owning one eighth of the matrix, so the dense operand rows a
// window needs are spread over the 8 L2s rather than replicated in time.  `hw_id` < a grid
// padded to a multiple of 8*block; ids >= the real count must be skipped by the caller.
__device__ __forceinline__ uint32_t xcd_block_cyclic_id(uint32_t hw_id, uint32_t block)
{
    const uint32_t xcd = hw_id % kXcds, j = hw_id / kXcds;
    return ((j / block) * kXcds + xcd) * block + j % block;
}

}  // namespace lapis
