// Batched GEMM for many small matrices, the batch dimension vectorised (Section 5 of the paper
// lowers this kernel as its example of a batched operation: the matrices are too small to be
// worth a tile each, so the lanes of a wavefront go across the batch).
// C[b] = alpha * A[b] * B[b] + beta * C[b], every matrix row-major, the matrices of an operand
// back to back (the layout of a contiguous (batch, rows, cols) tensor).
//
// One wavefront = one workgroup takes E consecutive batch entries (E a power of two, as many as
// fit in its LDS tile).  Their A and B matrices are one contiguous piece of memory each, which
// the wavefront streams into LDS with coalesced loads; P = 64 / E lanes then share one entry and
// each lane computes strips of 4 consecutive elements of a row of C out of LDS.  The kernel is
// bound by HBM (2 m n k flops for (m k + k n + m n [+ m n]) values), so everything is arranged
// around wide, contiguous global accesses.  Contracts of the entry point are in include/lapis.h.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <string>

#include "../../include/lapis.h"
#include "device_utils.hpp"
#include "internal.hpp"

namespace lapis {

constexpr int kGemmMaxDim = LAPIS_BATCHED_MAX_DIM;
// LDS tile of a wavefront: one entry of the largest size must fit, (2 * 32 * 32 + 1) doubles
constexpr int kGemmTileBytes = (2 * kGemmMaxDim * kGemmMaxDim + 1) * 8;
constexpr int kGemmStrip = 4;                        // consecutive elements of a row of C per work item

// floor(g / d) for 0 <= g < 2^20 and 1 <= d (inv = 1.0f / d): the float estimate is off by at
// most one either way
__device__ __forceinline__ uint32_t small_div(uint32_t g, uint32_t d, float inv)
{
    uint32_t q = (uint32_t)((float)g * inv);
    if (q * d > g) q -= 1;
    if ((q + 1) * d <= g) q += 1;
    return q;
}

// stride: LDS elements per entry (m*k + k*n, plus one if that is even: an odd stride keeps the
// lanes of different entries on different banks); entries_per_wave = E.
template <typename T>
__global__ __launch_bounds__(kWave) void batched_gemm_kernel(
    int64_t batch, int m, int n, int k, int entries_per_wave, int stride, T alpha, const T *__restrict__ A,
    const T *__restrict__ B, T beta, T *__restrict__ C)
{
    __shared__ __attribute__((aligned(16))) T s_tile[kGemmTileBytes / sizeof(T)];
    const int lane = threadIdx.x;
    const int E = entries_per_wave;
    const int P = kWave / E;
    const int64_t b0 = (int64_t)blockIdx.x * E;
    const int here = (int)(batch - b0 < E ? batch - b0 : E);       // entries of this tile
    const uint32_t mk = (uint32_t)(m * k), kn = (uint32_t)(k * n), mn = (uint32_t)(m * n);

    // stream the tile's A and B matrices into LDS: element g of the contiguous piece belongs to
    // entry g / mk (g / kn); 4 loads in flight per lane
    {
        const T *__restrict__ src = A + b0 * mk;
        const uint32_t count = (uint32_t)here * mk;
        const float inv = 1.0f / (float)mk;
        for (uint32_t g0 = 0; g0 < count; g0 += 4 * kWave) {         // uniform
            T v[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t g = g0 + q * kWave + lane;
                v[q] = load_stream(src + (g < count ? g : count - 1));
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t g = g0 + q * kWave + lane;
                if (g < count) {
                    const uint32_t e = small_div(g, mk, inv);
                    s_tile[e * stride + (g - e * mk)] = v[q];
                }
            }
        }
    }
    {
        const T *__restrict__ src = B + b0 * kn;
        const uint32_t count = (uint32_t)here * kn;
        const float inv = 1.0f / (float)kn;
        for (uint32_t g0 = 0; g0 < count; g0 += 4 * kWave) {         // uniform
            T v[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t g = g0 + q * kWave + lane;
                v[q] = load_stream(src + (g < count ? g : count - 1));
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t g = g0 + q * kWave + lane;
                if (g < count) {
                    const uint32_t e = small_div(g, kn, inv);
                    s_tile[e * stride + mk + (g - e * kn)] = v[q];
                }
            }
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // lane (e, p): work items p, p + P, ... of entry e; item w = (row i, strip of 4 columns)
    const int e = lane / P, p = lane % P;
    if (e >= here) return;
    const int strips = (n + kGemmStrip - 1) / kGemmStrip;
    const int items = m * strips;
    const float inv_strips = 1.0f / (float)strips;
    const T *a_lds = s_tile + e * stride;
    const T *b_lds = a_lds + mk;
    T *__restrict__ c_out = C + (b0 + e) * mn;
    for (int w = p; w < items; w += P) {
        const int i = (int)small_div((uint32_t)w, (uint32_t)strips, inv_strips);
        const int j0 = (w - i * strips) * kGemmStrip;
        // columns past n repeat column n - 1 and are not stored
        int col[kGemmStrip];
#pragma unroll
        for (int q = 0; q < kGemmStrip; ++q) col[q] = j0 + q < n ? j0 + q : n - 1;
        T acc[kGemmStrip];
#pragma unroll
        for (int q = 0; q < kGemmStrip; ++q) acc[q] = T(0);
        const T *a_row = a_lds + i * k;
        for (int l = 0; l < k; ++l) {
            const T a = a_row[l];
            const T *b_row = b_lds + l * n;
#pragma unroll
            for (int q = 0; q < kGemmStrip; ++q) acc[q] += a * b_row[col[q]];
        }
        T *dst = c_out + i * n + j0;
#pragma unroll
        for (int q = 0; q < kGemmStrip; ++q) {
            if (j0 + q < n) dst[q] = beta == T(0) ? alpha * acc[q] : alpha * acc[q] + beta * dst[q];
        }
    }
}

template <typename T>
int batched_gemm_typed(int64_t batch, int m, int n, int k, double alpha, const void *A, const void *B, double beta,
                       void *C, hipStream_t stream)
{
    int stride = m * k + k * n;
    if (stride % 2 == 0) stride += 1;
    const int capacity = kGemmTileBytes / (int)sizeof(T);
    int E = kWave;
    while (E > 1 && E * stride > capacity) E /= 2;
    const int64_t tiles = (batch + E - 1) / E;
    if (tiles > INT32_MAX) return fail(LAPIS_ERR_INVALID_ARG, "lapis_batched_gemm: batch is too large");
    batched_gemm_kernel<T><<<dim3((uint32_t)tiles), dim3(kWave), 0, stream>>>(
        batch, m, n, k, E, stride, (T)alpha, static_cast<const T *>(A), static_cast<const T *>(B), (T)beta,
        static_cast<T *>(C));
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess) return fail(LAPIS_ERR_DEVICE, std::string("lapis_batched_gemm: ") + hipGetErrorString(err));
    return LAPIS_OK;
}

}  // namespace lapis

extern "C" int lapis_batched_gemm(int64_t batch, int32_t m, int32_t n, int32_t k, double alpha, const void *d_A,
                                  const void *d_B, double beta, void *d_C, int dtype, void *hip_stream)
{
    using lapis::fail;
    if (batch < 0) return fail(LAPIS_ERR_INVALID_ARG, "lapis_batched_gemm: negative batch");
    if (m < 1 || n < 1 || k < 1 || m > LAPIS_BATCHED_MAX_DIM || n > LAPIS_BATCHED_MAX_DIM || k > LAPIS_BATCHED_MAX_DIM)
        return fail(LAPIS_ERR_INVALID_ARG, "lapis_batched_gemm: m, n and k must be between 1 and LAPIS_BATCHED_MAX_DIM");
    if (dtype != LAPIS_F32 && dtype != LAPIS_F64) return fail(LAPIS_ERR_UNSUPPORTED, "lapis_batched_gemm: dtype");
    if (batch == 0) return LAPIS_OK;
    if (!d_A || !d_B || !d_C) return fail(LAPIS_ERR_INVALID_ARG, "lapis_batched_gemm: NULL operand");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (dtype == LAPIS_F64) return lapis::batched_gemm_typed<double>(batch, m, n, k, alpha, d_A, d_B, beta, d_C, stream);
    return lapis::batched_gemm_typed<float>(batch, m, n, k, alpha, d_A, d_B, beta, d_C, stream);
}
