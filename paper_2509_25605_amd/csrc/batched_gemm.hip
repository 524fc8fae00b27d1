// Batched GEMM for many small matrices (Section 5 of the paper lowers this kernel as its example
// of a batched operation, with the batch dimension as the vectorised one).  Two kernels: for the
// small entries the lanes of a wavefront go across the batch (below); entries from about 12 x 12
// x 12 on get a wavefront each and the matrix cores (batched_gemm_mfma_kernel, further down).
// C[b] = alpha * A[b] * B[b] + beta * C[b], every matrix row-major, the matrices of an operand
// back to back (the layout of a contiguous (batch, rows, cols) tensor).
//
// One wavefront = one workgroup takes E consecutive batch entries (E a power of two, as many as
// fit in its LDS tile).  Their A and B matrices are one contiguous piece of memory each, which
// the wavefront streams into LDS with coalesced loads; P = 64 / E lanes then share one entry and
// each lane computes strips of 16 bytes (2 doubles, 4 floats) of a row of C out of LDS.  The kernel is
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
// LDS tile of a wavefront: one entry of the largest size must fit ((2 * 32 * 32 + 1) doubles), and
// 16 entries of 8 x 8 doubles with their padding (9 wavefronts per CU at that size)
constexpr int kGemmTileBytes = 2080 * 8;
static_assert(kGemmTileBytes >= (2 * kGemmMaxDim * kGemmMaxDim + 1) * 8, "one entry of the largest size must fit");
static_assert(kGemmMaxDim == 32, "the matrix-core path has at most 2 x 2 tiles of 16 x 16");
constexpr int kGemmMfmaMinElements = 400;   // elements of A, B and C of one entry from which the matrix cores take over
constexpr int kGemmMaxVec = (kGemmTileBytes / 16 + kWave - 1) / kWave;      // 16-byte loads per lane and tile

// floor(g / d) for 0 <= g < 2^20 and 1 <= d (inv = 1.0f / d): the float estimate is off by at
// most one either way
__device__ __forceinline__ uint32_t small_div(uint32_t g, uint32_t d, float inv)
{
    uint32_t q = (uint32_t)((float)g * inv);
    if (q * d > g) q -= 1;
    if ((q + 1) * d <= g) q += 1;
    return q;
}

// `count` consecutive elements from src into the tile: element g goes to entry g / d at offset
// shift + g % d; 4 loads in flight per lane (the path for tiles that are not full or not aligned)
template <typename T>
__device__ __forceinline__ void stage_scalar(const T *__restrict__ src, uint32_t count, uint32_t d, uint32_t shift,
                                             int stride, int lane, T *s_tile)
{
    const float inv = 1.0f / (float)d;
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
                const uint32_t e = small_div(g, d, inv);
                s_tile[e * stride + shift + (g - e * d)] = v[q];
            }
        }
    }
}

// stride: LDS elements per entry (m*k + k*n, plus one if that is even: an odd stride keeps the
// lanes of different entries on different banks); entries_per_wave = E.  VEC: the A and B pieces
// of a full tile are multiples of 16 bytes and A, B are 16-byte aligned.  VECC: every strip of C
// is 16 bytes at a 16-byte aligned address (C aligned, n a multiple of the strip).
// RB: rows of C per work item (a b value read from LDS serves RB products).  DIM > 0: m = n = k =
// DIM is known at compile time (loops unroll, divisions become multiplications, LDS offsets
// immediates); 0: the sizes are the run-time arguments.
template <typename T, bool VEC, bool VECC, int RB, int DIM = 0, bool DYN = false>
__global__ __launch_bounds__(kWave) void batched_gemm_kernel(
    int64_t batch, int m_arg, int n_arg, int k_arg, int entries_per_wave, int stride_arg, T alpha,
    const T *__restrict__ A, const T *__restrict__ B, T beta, T *__restrict__ C)
{
    const int m = DIM ? DIM : m_arg, n = DIM ? DIM : n_arg, k = DIM ? DIM : k_arg;
    const int stride = DIM ? (2 * DIM * DIM + 1) : stride_arg;
    constexpr int kGemmStrip = 16 / (int)sizeof(T);                // elements of a row of C per work item
    typedef T vec_t __attribute__((ext_vector_type(16 / sizeof(T))));
    // DYN: the launch sizes the tile to E * stride values, so tiny products leave room for more
    // wavefronts per CU; otherwise a fixed tile, whose addresses the compiler knows
    extern __shared__ __attribute__((aligned(16))) unsigned char s_tile_bytes[];
    __shared__ __attribute__((aligned(16))) T s_tile_fixed[DYN ? 1 : kGemmTileBytes / sizeof(T)];
    T *s_tile = DYN ? reinterpret_cast<T *>(s_tile_bytes) : s_tile_fixed;
    const int lane = threadIdx.x;
    const int E = entries_per_wave;
    const int P = kWave / E;
    const int64_t b0 = (int64_t)blockIdx.x * E;
    const int here = (int)(batch - b0 < E ? batch - b0 : E);       // entries of this tile
    const uint32_t mk = (uint32_t)(m * k), kn = (uint32_t)(k * n), mn = (uint32_t)(m * n);

    // stream the tile's A and B matrices into LDS: element g of the contiguous piece belongs to
    // entry g / mk (g / kn)
    if (VEC && here == E) {
        // a full tile whose pieces are multiples of 16 bytes at 16-byte aligned addresses (the host
        // checked): every 16-byte load of the tile is issued before the first value is stored
        constexpr int kPer = 16 / (int)sizeof(T);
        const uint32_t va = (uint32_t)E * mk / kPer, vb = (uint32_t)E * kn / kPer;
        const vec_t *__restrict__ src_a = reinterpret_cast<const vec_t *>(A + b0 * mk);
        const vec_t *__restrict__ src_b = reinterpret_cast<const vec_t *>(B + b0 * kn);
        const float inv_a = 1.0f / (float)mk, inv_b = 1.0f / (float)kn;
        const bool whole_a = mk % kPer == 0, whole_b = kn % kPer == 0;       // uniform
        vec_t v[kGemmMaxVec];
#pragma unroll
        for (int q = 0; q < kGemmMaxVec; ++q) {
            if ((uint32_t)(q * kWave) < va + vb) {                     // uniform
                uint32_t h = q * kWave + lane;
                h = h < va + vb ? h : va + vb - 1;
                v[q] = __builtin_nontemporal_load(h < va ? src_a + h : src_b + (h - va));
            }
        }
#pragma unroll
        for (int q = 0; q < kGemmMaxVec; ++q) {
            if ((uint32_t)(q * kWave) < va + vb) {
                const uint32_t h = q * kWave + lane;
                if (h < va + vb) {
                    const bool in_a = h < va;
                    const uint32_t d = in_a ? mk : kn, first = (in_a ? h : h - va) * kPer;
                    const float inv = in_a ? inv_a : inv_b;
                    const uint32_t shift = in_a ? 0 : mk;
                    if (whole_a && whole_b) {              // a vector never straddles two entries
                        const uint32_t e = DIM ? first / (uint32_t)(DIM * DIM) : small_div(first, d, inv);
                        T *dst = s_tile + e * stride + shift + (first - e * d);
#pragma unroll
                        for (int t = 0; t < kPer; ++t) dst[t] = v[q][t];
                    } else {
#pragma unroll
                        for (int t = 0; t < kPer; ++t) {
                            const uint32_t g = first + t;
                            const uint32_t e = small_div(g, d, inv);
                            s_tile[e * stride + shift + (g - e * d)] = v[q][t];
                        }
                    }
                }
            }
        }
    } else {
        stage_scalar(A + b0 * mk, (uint32_t)here * mk, mk, 0u, stride, lane, s_tile);
        stage_scalar(B + b0 * kn, (uint32_t)here * kn, kn, mk, stride, lane, s_tile);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // lane (e, p): work items p, p + P, ... of entry e; item w = (block of RB rows, strip of 16
    // bytes of them)
    const int e = lane / P, p = lane % P;
    if (e >= here) return;
    const int strips = (n + kGemmStrip - 1) / kGemmStrip;
    const int items = ((m + RB - 1) / RB) * strips;
    const float inv_strips = 1.0f / (float)strips;
    const T *a_lds = s_tile + e * stride;
    const T *b_lds = a_lds + mk;
    T *__restrict__ c_out = C + (b0 + e) * mn;
    for (int w = p; w < items; w += P) {
        const int ib = DIM ? w / (DIM / kGemmStrip) : (int)small_div((uint32_t)w, (uint32_t)strips, inv_strips);
        const int i0 = ib * RB;
        const int j0 = (w - ib * strips) * kGemmStrip;
        // rows past m repeat row m - 1, columns past n column n - 1; neither is stored
        int col[kGemmStrip];
#pragma unroll
        for (int q = 0; q < kGemmStrip; ++q) col[q] = j0 + q < n ? j0 + q : n - 1;
        const T *a_row[RB];
#pragma unroll
        for (int r = 0; r < RB; ++r) a_row[r] = a_lds + (i0 + r < m ? i0 + r : m - 1) * k;
        T acc[RB][kGemmStrip];
#pragma unroll
        for (int r = 0; r < RB; ++r)
#pragma unroll
            for (int q = 0; q < kGemmStrip; ++q) acc[r][q] = T(0);
        for (int l = 0; l < k; ++l) {
            const T *b_row = b_lds + l * n;
            T bv[kGemmStrip];
#pragma unroll
            for (int q = 0; q < kGemmStrip; ++q) bv[q] = b_row[col[q]];
#pragma unroll
            for (int r = 0; r < RB; ++r) {
                const T a = a_row[r][l];
#pragma unroll
                for (int q = 0; q < kGemmStrip; ++q) acc[r][q] += a * bv[q];
            }
        }
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            if (i0 + r < m) {
                T *dst = c_out + (i0 + r) * n + j0;
                if constexpr (VECC) {
                    vec_t out;
                    if (beta == T(0)) {
#pragma unroll
                        for (int q = 0; q < kGemmStrip; ++q) out[q] = alpha * acc[r][q];
                    } else {
                        const vec_t old = *reinterpret_cast<const vec_t *>(dst);
#pragma unroll
                        for (int q = 0; q < kGemmStrip; ++q) out[q] = alpha * acc[r][q] + beta * old[q];
                    }
                    *reinterpret_cast<vec_t *>(dst) = out;
                } else {
#pragma unroll
                    for (int q = 0; q < kGemmStrip; ++q) {
                        if (j0 + q < n) dst[q] = beta == T(0) ? alpha * acc[r][q] : alpha * acc[r][q] + beta * dst[q];
                    }
                }
            }
        }
    }
}

// Matrices whose sides are multiples of the 16 x 16 x 4 matrix-core tile: one wavefront per batch
// entry (kWavesPerBlock of them in a workgroup), no LDS.  Every lane loads its fragments of A (16 bytes = H consecutive k of one row) and
// of B (one element of H rows) straight from memory, all loads of the entry in flight together;
// lane (i, g) = (lane % 16, lane / 16) supplies A[16 rt + i][kk] and B[kk][16 ct + i] with
// kk = 4 H q + H g + h for the instruction (q, h) - the k index only has to agree between the
// two operands, so it is chosen to make A's loads 16 bytes wide.  Each matrix element is read
// once.  M = 16 MT, N = 16 NT, K = 4 H KQ; A 16-byte aligned.
template <typename T> struct MfmaTile;
template <> struct MfmaTile<double> {
    typedef double acc_t __attribute__((ext_vector_type(4)));
    static __device__ __forceinline__ acc_t mma(double a, double b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
    }
    // row of the tile that register v of lane group g holds (the column is lane % 16)
    static __device__ __forceinline__ int row(int g, int v) { return g + 4 * v; }
};
template <> struct MfmaTile<float> {
    typedef float acc_t __attribute__((ext_vector_type(4)));
    static __device__ __forceinline__ acc_t mma(float a, float b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int row(int g, int v) { return 4 * g + v; }
};

// MODE 2 (exact): m = 16 MT, n = 16 NT, k = 4 H KQ and A is 16-byte aligned.  Otherwise those are
// the sizes rounded up: elements outside the matrices are not loaded and count as zeros (rows of
// C past m and columns past n may then pick up anything, they are not stored).  MODE 1: k is a
// multiple of H and A 16-byte aligned, so A's 16-byte pieces are whole and aligned; MODE 0: A is
// read element by element.
template <typename T, int MT, int NT, int KQ, int MODE>
__global__ __launch_bounds__(kBlock) void batched_gemm_mfma_kernel(int64_t batch, int m_arg, int n_arg, int k_arg,
                                                                   T alpha, const T *__restrict__ A,
                                                                   const T *__restrict__ B, T beta, T *__restrict__ C)
{
    constexpr int H = 16 / (int)sizeof(T);
    constexpr bool EXACT = MODE == 2;
    const int m = EXACT ? 16 * MT : m_arg, n = EXACT ? 16 * NT : n_arg, k = EXACT ? 4 * H * KQ : k_arg;
    typedef T vec_t __attribute__((ext_vector_type(16 / sizeof(T))));
    typedef typename MfmaTile<T>::acc_t acc_t;
    const int lane = threadIdx.x % kWave, i = lane % 16, g = lane / 16;
    const int64_t b = (int64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
    if (b >= batch) return;                              // whole wavefronts leave together
    const T *__restrict__ a = A + b * (m * k);
    const T *__restrict__ bm = B + b * (k * n);
    T *__restrict__ c = C + b * (m * n);
    vec_t af[MT][KQ];
    T bf[KQ][H][NT];
#pragma unroll
    for (int rt = 0; rt < MT; ++rt)
#pragma unroll
        for (int q = 0; q < KQ; ++q) {
            const int row = rt * 16 + i, kk = q * 4 * H + g * H;
            if constexpr (EXACT) {
                af[rt][q] = *reinterpret_cast<const vec_t *>(a + row * k + kk);
            } else if constexpr (MODE == 1) {
                vec_t zero;
#pragma unroll
                for (int h = 0; h < H; ++h) zero[h] = T(0);
                af[rt][q] = (row < m && kk < k) ? *reinterpret_cast<const vec_t *>(a + row * k + kk) : zero;
            } else {
#pragma unroll
                for (int h = 0; h < H; ++h) af[rt][q][h] = (row < m && kk + h < k) ? a[row * k + kk + h] : T(0);
            }
        }
#pragma unroll
    for (int q = 0; q < KQ; ++q)
#pragma unroll
        for (int h = 0; h < H; ++h)
#pragma unroll
            for (int ct = 0; ct < NT; ++ct) {
                // 16 doubles are a whole 128-byte line, read by nobody else; 16 floats share their
                // line with another load of this wavefront (and so do A's 16 bytes per lane)
                const int kk = q * 4 * H + g * H + h, col = ct * 16 + i;
                const T *src = bm + kk * n + col;
                if constexpr (EXACT) bf[q][h][ct] = sizeof(T) == 8 ? __builtin_nontemporal_load(src) : *src;
                else bf[q][h][ct] = (kk < k && col < n) ? *src : T(0);
            }
    acc_t acc[MT][NT];
#pragma unroll
    for (int rt = 0; rt < MT; ++rt)
#pragma unroll
        for (int ct = 0; ct < NT; ++ct) acc[rt][ct] = acc_t{0, 0, 0, 0};
#pragma unroll
    for (int q = 0; q < KQ; ++q)
#pragma unroll
        for (int h = 0; h < H; ++h)
#pragma unroll
            for (int rt = 0; rt < MT; ++rt)
#pragma unroll
                for (int ct = 0; ct < NT; ++ct) acc[rt][ct] = MfmaTile<T>::mma(af[rt][q][h], bf[q][h][ct], acc[rt][ct]);
#pragma unroll
    for (int rt = 0; rt < MT; ++rt)
#pragma unroll
        for (int ct = 0; ct < NT; ++ct)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = rt * 16 + MfmaTile<T>::row(g, v), col = ct * 16 + i;
                if (EXACT || (row < m && col < n)) {
                    T *dst = c + row * n + col;
                    *dst = beta == T(0) ? alpha * acc[rt][ct][v] : alpha * acc[rt][ct][v] + beta * *dst;
                }
            }
}

template <typename T>
int batched_gemm_typed(int64_t batch, int m, int n, int k, double alpha, const void *A, const void *B, double beta,
                       void *C, hipStream_t stream)
{
    // entries of kGemmMfmaMinElements and more go to the matrix cores, one wavefront per entry
    // (measured: 12 x 12 x 12 and up are faster there, 8 x 8 x 8 and 10 x 20 x 5 are not)
    if (m * k + k * n + m * n >= kGemmMfmaMinElements) {
        constexpr int kStep = 4 * (16 / (int)sizeof(T));
        constexpr int kMaxKq = kGemmMaxDim / kStep;
        if (batch > INT32_MAX) return fail(LAPIS_ERR_INVALID_ARG, "lapis_batched_gemm: batch is too large");
        const int mt = (m + 15) / 16, nt = (n + 15) / 16, kq = (k + kStep - 1) / kStep;
        const bool aligned = reinterpret_cast<uintptr_t>(A) % 16 == 0;
        const bool exact = m % 16 == 0 && n % 16 == 0 && k % kStep == 0 && aligned;
        const bool whole = k % (kStep / 4) == 0 && aligned;       // A's 16-byte pieces
#define LAPIS_GEMM_MFMA(MT, NT, KQ, MODE)                                                                        \
    batched_gemm_mfma_kernel<T, MT, NT, KQ, MODE>                                                                \
        <<<dim3((uint32_t)((batch + kWavesPerBlock - 1) / kWavesPerBlock)), dim3(kBlock), 0, stream>>>(          \
            batch, m, n, k, (T)alpha, static_cast<const T *>(A), static_cast<const T *>(B), (T)beta, static_cast<T *>(C))
#define LAPIS_GEMM_MFMA_E(MT, NT, KQ)                    \
    do {                                                 \
        if (exact) LAPIS_GEMM_MFMA(MT, NT, KQ, 2);       \
        else if (whole) LAPIS_GEMM_MFMA(MT, NT, KQ, 1);  \
        else LAPIS_GEMM_MFMA(MT, NT, KQ, 0);             \
    } while (0)
        // kq <= kMaxKq (2 for floats, 4 for doubles); the clamps keep the other cases from being built
#define LAPIS_GEMM_MFMA_K(MT, NT)                                                        \
    do {                                                                                 \
        if (kq == 1) LAPIS_GEMM_MFMA_E(MT, NT, 1);                                       \
        else if (kq == 2) LAPIS_GEMM_MFMA_E(MT, NT, 2);                                  \
        else if (kq == 3) LAPIS_GEMM_MFMA_E(MT, NT, (kMaxKq >= 3 ? 3 : 1));              \
        else LAPIS_GEMM_MFMA_E(MT, NT, (kMaxKq >= 4 ? 4 : 1));                           \
    } while (0)
        if (mt == 1 && nt == 1) LAPIS_GEMM_MFMA_K(1, 1);
        else if (mt == 1) LAPIS_GEMM_MFMA_K(1, 2);
        else if (nt == 1) LAPIS_GEMM_MFMA_K(2, 1);
        else LAPIS_GEMM_MFMA_K(2, 2);
#undef LAPIS_GEMM_MFMA_K
#undef LAPIS_GEMM_MFMA_E
#undef LAPIS_GEMM_MFMA
        const hipError_t err = hipGetLastError();
        if (err != hipSuccess) return fail(LAPIS_ERR_DEVICE, std::string("lapis_batched_gemm: ") + hipGetErrorString(err));
        return LAPIS_OK;
    }
    int stride = m * k + k * n;
    if (stride % 2 == 0) stride += 1;
    const int capacity = kGemmTileBytes / (int)sizeof(T);
    int E = kWave;
    while (E > 1 && E * stride > capacity) E /= 2;
    const int64_t tiles = (batch + E - 1) / E;
    const size_t lds_bytes = ((size_t)E * stride * sizeof(T) + 15) / 16 * 16;
    const bool tiny = lds_bytes <= 8192;          // at least twice the wavefronts per CU of the fixed tile
    if (tiles > INT32_MAX) return fail(LAPIS_ERR_INVALID_ARG, "lapis_batched_gemm: batch is too large");
    const bool vec = reinterpret_cast<uintptr_t>(A) % 16 == 0 && reinterpret_cast<uintptr_t>(B) % 16 == 0 &&
                     ((size_t)E * m * k * sizeof(T)) % 16 == 0 && ((size_t)E * k * n * sizeof(T)) % 16 == 0;
    const int strip = 16 / (int)sizeof(T);
    const bool vecc = reinterpret_cast<uintptr_t>(C) % 16 == 0 && n % strip == 0;
    // blocks of 4 rows per work item when that still leaves every lane of an entry an item
    const int P = kWave / E;
    const bool blocked = ((m + 3) / 4) * ((n + strip - 1) / strip) >= P;
#define LAPIS_GEMM_LAUNCH(VEC, VECC, RB)                                                                        \
    do {                                                                                                        \
        if (tiny)                                                                                               \
            batched_gemm_kernel<T, VEC, VECC, RB, 0, true><<<dim3((uint32_t)tiles), dim3(kWave), lds_bytes, stream>>>( \
                batch, m, n, k, E, stride, (T)alpha, static_cast<const T *>(A), static_cast<const T *>(B),      \
                (T)beta, static_cast<T *>(C));                                                                  \
        else                                                                                                    \
            batched_gemm_kernel<T, VEC, VECC, RB><<<dim3((uint32_t)tiles), dim3(kWave), 0, stream>>>(           \
                batch, m, n, k, E, stride, (T)alpha, static_cast<const T *>(A), static_cast<const T *>(B),      \
                (T)beta, static_cast<T *>(C));                                                                  \
    } while (0)
#define LAPIS_GEMM_PICK(VEC, VECC)                       \
    do {                                                 \
        if (blocked) LAPIS_GEMM_LAUNCH(VEC, VECC, 4);    \
        else LAPIS_GEMM_LAUNCH(VEC, VECC, 1);            \
    } while (0)
    const bool cube = m == n && n == k && vec && vecc && blocked;
#define LAPIS_GEMM_CUBE(D)                                                                                      \
    batched_gemm_kernel<T, true, true, 4, D><<<dim3((uint32_t)tiles), dim3(kWave), 0, stream>>>(                \
        batch, m, n, k, E, stride, (T)alpha, static_cast<const T *>(A), static_cast<const T *>(B), (T)beta,     \
        static_cast<T *>(C))
    if (cube && m == 4)
        batched_gemm_kernel<T, true, true, 4, 4, true><<<dim3((uint32_t)tiles), dim3(kWave), lds_bytes, stream>>>(
            batch, m, n, k, E, stride, (T)alpha, static_cast<const T *>(A), static_cast<const T *>(B), (T)beta,
            static_cast<T *>(C));
    else if (cube && m == 8) LAPIS_GEMM_CUBE(8);
    else if (vec && vecc) LAPIS_GEMM_PICK(true, true);
    else if (vec) LAPIS_GEMM_PICK(true, false);
    else if (vecc) LAPIS_GEMM_PICK(false, true);
    else LAPIS_GEMM_PICK(false, false);
#undef LAPIS_GEMM_CUBE
#undef LAPIS_GEMM_PICK
#undef LAPIS_GEMM_LAUNCH
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
