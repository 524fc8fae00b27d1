// Measurement kernels behind include/lapis_ceilings.h: what one MI355X delivers for a plain
// streaming read, for random 8-byte gathers and for 128-byte rows pulled through the L1 of every
// CU.  bench.py times them beside the products; they are not part of the product library.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/lapis_ceilings.h"

namespace {

typedef double d2v __attribute__((ext_vector_type(2)));
constexpr int kThreads = 256;
constexpr int kPerThread = 4;       // 16-byte loads in flight per lane (read), 8 gathers (gather)

// Workgroup b reads the contiguous piece [b * 256 * 4, (b + 1) * 256 * 4) of 16-byte items, all
// loads issued before the first use: the shape of a wavefront streaming its chunk of a matrix.
template <bool NT>
__global__ __launch_bounds__(kThreads) void read_kernel(const d2v *__restrict__ p, int64_t n16, double *sink)
{
    const int64_t base = (int64_t)blockIdx.x * kThreads * kPerThread + threadIdx.x;
    d2v v[kPerThread];
#pragma unroll
    for (int u = 0; u < kPerThread; ++u) {
        const int64_t i = base + u * kThreads;
        v[u] = i < n16 ? (NT ? __builtin_nontemporal_load(p + i) : p[i]) : d2v{0, 0};
    }
    double s = 0;
#pragma unroll
    for (int u = 0; u < kPerThread; ++u) s += v[u].x + v[u].y;
    if (s == 1.2345e300) sink[0] = s;
}

__global__ __launch_bounds__(kThreads) void gather_kernel(const double *__restrict__ x, int64_t len,
                                                         const int32_t *__restrict__ idx, int64_t n, double *sink)
{
    constexpr int U = 8;
    const int64_t i = (int64_t)blockIdx.x * kThreads * U + threadIdx.x;
    int32_t c[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int32_t j = (i + u * kThreads < n) ? __builtin_nontemporal_load(idx + i + u * kThreads) : 0;
        c[u] = (j >= 0 && j < len) ? j : 0;
    }
    double s = 0;
#pragma unroll
    for (int u = 0; u < U; ++u) s += x[c[u]];
    if (s == 1.2345e300) sink[0] = s;
}

// Lane l of group g (8 lanes) reads bytes 16 l .. 16 l + 15 of a row; 16 rows in flight per lane.
// The row numbers come from a generator in registers, so nothing but the rows is loaded.
__global__ __launch_bounds__(64) void rows_kernel(const double *__restrict__ table, uint32_t row_mask, int iters,
                                                  int random, double *sink)
{
    constexpr int kInFlight = 16;
    const int lane = threadIdx.x, grp = lane / 8, l = lane % 8;
    uint32_t state = blockIdx.x * 2654435761u + 12345u;      // the same in every lane of the wavefront
    d2v acc = {0, 0};
    for (int it = 0; it < iters; ++it) {
        d2v v[kInFlight];
#pragma unroll
        for (int t = 0; t < kInFlight; ++t) {
            state = state * 1664525u + 1013904223u;
            uint32_t r = random ? ((state >> 8) * (2 * grp + 1) + grp * 7919u) : ((state >> 8) + grp);
            r &= row_mask;
            v[t] = *reinterpret_cast<const d2v *>(table + (size_t)r * 16 + l * 2);
        }
#pragma unroll
        for (int t = 0; t < kInFlight; ++t) acc += v[t];
    }
    if (acc[0] + acc[1] == 1.2345e300) sink[0] = acc[0];
}

}  // namespace

extern "C" {

int lapis_ceiling_read(const void *d_buf, int64_t bytes, int nontemporal, void *d_sink, void *hip_stream)
{
    if (!d_buf || !d_sink || bytes <= 0 || bytes % 16 != 0 || reinterpret_cast<uintptr_t>(d_buf) % 16 != 0) return 1;
    const int64_t n16 = bytes / 16;
    const int64_t blocks = (n16 + kThreads * kPerThread - 1) / (kThreads * kPerThread);
    if (blocks > 0x7fffffff) return 1;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (nontemporal)
        read_kernel<true><<<dim3((uint32_t)blocks), dim3(kThreads), 0, s>>>(static_cast<const d2v *>(d_buf), n16,
                                                                            static_cast<double *>(d_sink));
    else
        read_kernel<false><<<dim3((uint32_t)blocks), dim3(kThreads), 0, s>>>(static_cast<const d2v *>(d_buf), n16,
                                                                             static_cast<double *>(d_sink));
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int lapis_ceiling_gather(const double *d_table, int64_t table_len, const int32_t *d_idx, int64_t n, void *d_sink,
                         void *hip_stream)
{
    if (!d_table || !d_idx || !d_sink || table_len <= 0 || table_len > 0x7fffffff || n <= 0) return 1;
    const int64_t blocks = (n + kThreads * 8 - 1) / (kThreads * 8);
    if (blocks > 0x7fffffff) return 1;
    gather_kernel<<<dim3((uint32_t)blocks), dim3(kThreads), 0, static_cast<hipStream_t>(hip_stream)>>>(
        d_table, table_len, d_idx, n, static_cast<double *>(d_sink));
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int lapis_ceiling_rows(const double *d_table, int64_t table_rows, int32_t iters, int32_t num_waves, int random,
                       void *d_sink, void *hip_stream)
{
    if (!d_table || !d_sink || table_rows <= 0 || (table_rows & (table_rows - 1)) != 0 || table_rows > (1ll << 31) ||
        iters <= 0 || num_waves <= 0)
        return 1;
    rows_kernel<<<dim3((uint32_t)num_waves), dim3(64), 0, static_cast<hipStream_t>(hip_stream)>>>(
        d_table, (uint32_t)(table_rows - 1), iters, random, static_cast<double *>(d_sink));
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

}  // extern "C"
