// C ABI of the gfx950 CSR SpMV / SpMM library: argument checks, the handle,
// the analysis driver and the kernel launches.  Declarations and the contract
// of every entry point are in include/lapis.h.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>

#include "transpose_kernels.hpp"
#include "radix_transpose_kernels.hpp"
#include "internal.hpp"
#include "../../include/lapis.h"
#include "analysis_kernels.hpp"
#include "spmm_kernels.hpp"
#include "spmv_kernels.hpp"

using namespace lapis;

static_assert(LAPIS_NUM_BINS == kNumBins, "header and kernels disagree on the bin count");
static_assert(LAPIS_WAVE == kWave, "header and kernels disagree on the wavefront width");
static_assert(LAPIS_LONG_THRESHOLD >= LAPIS_TILE_NNZ, "a tile must touch at most two rows");
static_assert(LAPIS_TILE_NNZ % kBlock == 0, "tile size must be a multiple of the workgroup size");
static_assert(LAPIS_STREAM_ROWS == kStreamRows, "header and kernels disagree on the stream chunk size");
static_assert(LAPIS_STREAM_ROWS * LAPIS_WAVE <= 3 * kStreamWindow - 4, "a stream chunk must fit in three LDS windows");

namespace {

// A set of rows (the matrix's own rows outside stream chunks, or the virtual rows of the column
// split) partitioned into bins, plus the tile table of its last bin.  Row i of the set owns the
// entries row_begin[i] .. row_end[i] - 1.
struct BinnedSet {
    int64_t num_rows = 0;            // rows offered to the binning (before stream chunks are skipped)
    const int32_t *row_begin = nullptr;
    const int32_t *row_end = nullptr;
    int32_t *d_bin_offset = nullptr; // [kNumBins + 1]
    int32_t *d_row_perm = nullptr;   // [num_binned], allocated for num_rows
    int32_t *d_long_off = nullptr;   // [num_long + 1]
    int32_t *d_tile_row = nullptr;   // [num_tiles + 1]
    int32_t *d_tile_nz = nullptr;    // [num_tiles + 1]
    void *d_partial = nullptr;       // [2 * num_tiles] of the value type: per-tile segment sums
    int32_t h_bin_offset[kNumBins + 1] = {0};
    int64_t num_binned = 0, num_long = 0, num_tiles = 0;
};

}  // namespace

struct lapis_csr {
    int64_t nrows = 0, ncols = 0, nnz = 0;
    int dtype = 0;
    const int32_t *rowptr = nullptr;
    const int32_t *colidx = nullptr;
    const void *vals = nullptr;
    // arrays the handle owns (a transposed handle's CSR arrays); null when the arrays are borrowed
    int32_t *own_rowptr = nullptr, *own_colidx = nullptr;
    void *own_vals = nullptr;
    // level 1: stream chunks
    int32_t *d_stream_chunks = nullptr;  // [num_stream] chunk ids, class by class, ascending in a class
    int32_t h_stream_offset[kStreamClasses + 1] = {0};   // class boundaries in that list
    int64_t num_chunks = 0, num_stream = 0;
    int64_t half_bandwidth = 0;          // max |column - row| over the entries
    // level 1b: 16-bit column offsets of the stream chunks whose columns span less than 2^16
    int32_t *d_chunk_base = nullptr;     // [num_chunks] smallest column of such a chunk, else -1; null: off
    uint16_t *d_col16 = nullptr;         // [nnz rounded up to 8, + 8] colidx[j] - base of j's chunk
    int32_t *d_frame_table = nullptr;    // [32 * num_chunks] frames of the framed chunks (chunk_base == -2)
    int64_t narrow_entries = 0;          // entries in the chunks that could get a base
    int64_t framed_entries = 0;          // entries in the chunks that got a frame table instead
    bool class_all16[kStreamClasses] = {false, false, false, false};   // every chunk of the class has a base
    bool class_allframed[kStreamClasses] = {false, false, false, false};   // every chunk of the class is framed
    bool class_allcoded[kStreamClasses] = {false, false, false, false};    // every chunk is one or the other
    bool scattered_columns = false;      // few entries continue a run of consecutive columns (see launch_stream)
    // level 1c: row patterns (kept when the patterned chunks hold at least half of the entries)
    int32_t *d_pat_off = nullptr;        // [num_chunks + 1] exclusive scan of the chunks' table lengths
    uint16_t *d_row_pat = nullptr;       // [nrows] start of the row's pattern in its chunk's table
    int32_t *d_pat_pool = nullptr;       // the tables back to back
    int64_t pattern_entries = 0;         // entries in patterned chunks
    int64_t pattern_pool = 0;            // diagonals in the pool
    bool class_allpattern[kStreamClasses] = {false, false, false, false};  // every chunk of the class is patterned
    bool class_pattern16[kStreamClasses] = {false, false, false, false};   // ... is patterned, narrow or framed
    // SpMM: the stream chunks whose neighbouring rows share rows of X (spmm_share_flag_kernel), then the others
    int32_t *d_spmm_chunks = nullptr;    // [num_stream]; null when no chunk shares rows
    int32_t *d_share_flag = nullptr;     // [num_chunks] 1: shares rows, 2: another stream chunk, 0: not a stream chunk
    int32_t h_spmm_offset[kChunkClasses + 1] = {0};   // lists of the share classes 1..4 (kSharePlain, kShareNone, kShareBlock3, kShareBlock2)
    // level 2: bins over the rows outside stream chunks
    BinnedSet rows;
    // column split of the rows of bins 8-9 into virtual rows (num_blocks == 0: off)
    int64_t num_blocks = 0, block_width = 0, num_split = 0;
    int32_t *d_split_rows = nullptr;     // [num_split] rows of bins 8-9 with at most LAPIS_HUGE_ROW entries
    int32_t *d_cut = nullptr;            // [(num_blocks + 1) * num_split]
    void *d_vsum = nullptr;              // [num_blocks * num_split] of the value type
    BinnedSet vrows;
    // rows of more than LAPIS_HUGE_ROW entries, cut at LDS-sized column blocks (only with the split on)
    int64_t num_huge = 0, num_fblocks = 0, fblock_width = 0;
    int32_t *d_huge_rows = nullptr;      // [num_huge]
    int32_t *d_fcut = nullptr;           // [(num_fblocks + 1) * num_huge]
    void *d_fsum = nullptr;              // [num_fblocks * num_huge] of the value type
    // launch plans for spmv_short_kernel
    ShortPlan plan_rows;       // bins 0..8 of `rows` (0..7 when the split is on)
    ShortPlan plan_vrows;      // bins 0..8 of `vrows`
    // Products that use the handle's scratch (tile sums, virtual-row sums, block sums) are ordered among
    // themselves: each records scratch_event on its stream, and one that is enqueued on another stream
    // than the last first makes its stream wait for that event.  Null when the handle has no scratch.
    mutable std::mutex scratch_lock;
    mutable hipEvent_t scratch_event = nullptr;
    mutable hipStream_t scratch_stream = nullptr;
    mutable bool scratch_used = false;
};

namespace {
thread_local std::string g_last_error;
}

// Scratch of lapis_spmv_static_scratch: lives in the code object, one copy per GPU the library
// runs on, held until the process ends.  In host code the name below is only a stand-in for the
// symbol; its device address comes from hipGetSymbolAddress (static_scratch_address) and that
// address, never the name, is what kernels and copies get.
static __device__ __align__(256) unsigned char scratch[LAPIS_STATIC_SCRATCH_BYTES];

int lapis::fail(int code, const std::string &msg)
{
    g_last_error = msg;
    return code;
}

void lapis::vector_bytes(const lapis_csr *A, int64_t *x_bytes, int64_t *y_bytes)
{
    const int64_t esize = A->dtype == LAPIS_F64 ? 8 : 4;
    *x_bytes = A->ncols * esize;
    *y_bytes = A->nrows * esize;
}

namespace {

using lapis::fail;

int fail_hip(hipError_t e, const char *what)
{
    return fail(e == hipErrorOutOfMemory ? LAPIS_ERR_ALLOC : LAPIS_ERR_DEVICE,
                std::string(what) + ": " + hipGetErrorString(e));
}

#define LAPIS_STR2(x) #x
#define LAPIS_STR(x) LAPIS_STR2(x)
#define LAPIS_HIP(call)                                        \
    do {                                                       \
        hipError_t e_ = (call);                                \
        if (e_ != hipSuccess) return fail_hip(e_, #call " (lapis_api.hip:" LAPIS_STR(__LINE__) ")"); \
    } while (0)

template <typename P>
int device_alloc(P **ptr, size_t bytes)
{
    void *p = nullptr;
    hipError_t e = hipMalloc(&p, bytes ? bytes : 1);
    if (e != hipSuccess) return fail_hip(e, "hipMalloc");
    *ptr = static_cast<P *>(p);
    return LAPIS_OK;
}

// Small device-to-host readback through a pinned staging buffer (a copy into pageable memory
// costs a few hundred microseconds), followed by a stream synchronisation.  One buffer per host
// thread, allocated on first use and kept for the life of the process.
int read_back(void *dst, const void *d_src, size_t bytes, hipStream_t stream)
{
    constexpr size_t kStageBytes = 256;
    thread_local void *stage = nullptr;
    if (bytes > kStageBytes) return fail(LAPIS_ERR_DEVICE, "readback larger than the staging buffer");
    if (!stage) {
        hipError_t e = hipHostMalloc(&stage, kStageBytes, hipHostMallocDefault);
        if (e != hipSuccess) { stage = nullptr; return fail_hip(e, "hipHostMalloc"); }
    }
    LAPIS_HIP(hipMemcpyAsync(stage, d_src, bytes, hipMemcpyDeviceToHost, stream));
    LAPIS_HIP(hipStreamSynchronize(stream));
    std::memcpy(dst, stage, bytes);
    return LAPIS_OK;
}

// Frees on scope exit; for the temporaries of the analysis.
struct DeviceTemp {
    void *p = nullptr;
    ~DeviceTemp() { (void)hipFree(p); }
    template <typename P> P *as() { return static_cast<P *>(p); }
    int alloc(size_t bytes) { return device_alloc(&p, bytes); }
};

// hipFree that remembers the first failure (a pointer freed twice or never allocated here would
// otherwise surface later, as the "last error" of an unrelated call).
struct Freer {
    hipError_t first = hipSuccess;
    const char *what = nullptr;
    void operator()(void *p, const char *name)
    {
        const hipError_t e = hipFree(p);
        if (e != hipSuccess && first == hipSuccess) { first = e; what = name; }
    }
};
#define LAPIS_FREE(f, p) f((void *)(p), #p)

void free_set(BinnedSet &s, Freer &f)
{
    LAPIS_FREE(f, s.d_bin_offset);
    LAPIS_FREE(f, s.d_row_perm);
    LAPIS_FREE(f, s.d_long_off);
    LAPIS_FREE(f, s.d_tile_row);
    LAPIS_FREE(f, s.d_tile_nz);
    LAPIS_FREE(f, s.d_partial);
}

int free_handle(lapis_csr *A)
{
    if (!A) return LAPIS_OK;
    Freer f;
    LAPIS_FREE(f, A->d_stream_chunks);
    LAPIS_FREE(f, A->d_cut);
    LAPIS_FREE(f, A->d_split_rows);
    LAPIS_FREE(f, A->d_huge_rows);
    LAPIS_FREE(f, A->d_fcut);
    LAPIS_FREE(f, A->d_fsum);
    LAPIS_FREE(f, A->d_vsum);
    LAPIS_FREE(f, A->d_chunk_base);
    LAPIS_FREE(f, A->d_col16);
    LAPIS_FREE(f, A->d_frame_table);
    LAPIS_FREE(f, A->d_pat_off);
    LAPIS_FREE(f, A->d_row_pat);
    LAPIS_FREE(f, A->d_pat_pool);
    LAPIS_FREE(f, A->d_spmm_chunks);
    LAPIS_FREE(f, A->d_share_flag);
    LAPIS_FREE(f, A->own_rowptr);
    LAPIS_FREE(f, A->own_colidx);
    LAPIS_FREE(f, A->own_vals);
    free_set(A->rows, f);
    free_set(A->vrows, f);
    if (A->scratch_event) {
        const hipError_t e = hipEventDestroy(A->scratch_event);
        if (e != hipSuccess && f.first == hipSuccess) { f.first = e; f.what = "hipEventDestroy(scratch_event)"; }
    }
    delete A;
    if (f.first != hipSuccess) return fail_hip(f.first, f.what);
    return LAPIS_OK;
}

size_t value_size(const lapis_csr *A) { return A->dtype == LAPIS_F64 ? sizeof(double) : sizeof(float); }

// Workgroup ranges of bins 0..last_bin of a set; every bin is padded to a multiple of the XCD count.
void build_short_plan(const BinnedSet &s, int last_bin, ShortPlan *p)
{
    uint32_t blocks = 0;
    for (int b = 0; b < kShortBins; ++b) {
        p->bin_begin[b] = s.h_bin_offset[b];
        p->bin_count[b] = (b <= last_bin) ? s.h_bin_offset[b + 1] - s.h_bin_offset[b] : 0;
        p->block_begin[b] = blocks;
        const int per_block = short_rows_per_block(b);
        const uint32_t need = (uint32_t)(((int64_t)p->bin_count[b] + per_block - 1) / per_block);
        blocks += (need + kXcds - 1) / kXcds * kXcds;
    }
    p->block_begin[kShortBins] = blocks;
    p->num_blocks = blocks;
}

// Bins, stable row lists and the tile table of a row set.  chunk_flag (may be null) marks the
// chunks whose rows are left out.  Synchronises the stream.
int bin_row_set(BinnedSet *s, const int32_t *d_chunk_flag, size_t esize, hipStream_t stream)
{
    const int64_t n = s->num_rows;
    if (int rc = device_alloc(&s->d_bin_offset, sizeof(int32_t) * (kNumBins + 1))) return rc;
    if (int rc = device_alloc(&s->d_row_perm, sizeof(int32_t) * (size_t)n)) return rc;
    LAPIS_HIP(hipMemsetAsync(s->d_bin_offset, 0, sizeof(int32_t) * (kNumBins + 1), stream));
    if (n > 0) {
        const int32_t num_blocks = (int32_t)((n + kRowsPerAnalysisBlock - 1) / kRowsPerAnalysisBlock);
        DeviceTemp hist;
        if (int rc = hist.alloc(sizeof(int32_t) * (size_t)kNumBins * num_blocks)) return rc;
        bin_count_kernel<LAPIS_LONG_THRESHOLD><<<dim3(num_blocks), dim3(kBlock), 0, stream>>>(
            (int32_t)n, s->row_begin, s->row_end, LAPIS_STREAM_ROWS, d_chunk_flag, num_blocks, hist.as<int32_t>());
        bin_scan_kernel<<<dim3(1), dim3(kBlock), 0, stream>>>((int64_t)kNumBins * num_blocks, num_blocks,
                                                              hist.as<int32_t>(), s->d_bin_offset);
        bin_scatter_kernel<LAPIS_LONG_THRESHOLD><<<dim3(num_blocks), dim3(kBlock), 0, stream>>>(
            (int32_t)n, s->row_begin, s->row_end, LAPIS_STREAM_ROWS, d_chunk_flag, num_blocks,
            hist.as<int32_t>(), s->d_row_perm);
        LAPIS_HIP(hipGetLastError());
        if (int rc = read_back(s->h_bin_offset, s->d_bin_offset, sizeof(int32_t) * (kNumBins + 1), stream)) return rc;
    }
    s->num_binned = s->h_bin_offset[kNumBins];

    // long rows: scan of their lengths, then the tile table
    const int32_t m = s->h_bin_offset[kNumBins] - s->h_bin_offset[kNumBins - 1];
    s->num_long = m;
    if (int rc = device_alloc(&s->d_long_off, sizeof(int32_t) * ((size_t)m + 1))) return rc;
    int32_t long_total = 0;
    if (m > 0) {
        long_scan_kernel<<<dim3(1), dim3(kBlock), 0, stream>>>(
            m, s->d_row_perm + s->h_bin_offset[kNumBins - 1], s->row_begin, s->row_end, s->d_long_off);
        if (int rc = read_back(&long_total, s->d_long_off + m, sizeof(int32_t), stream)) return rc;
    } else {
        LAPIS_HIP(hipMemsetAsync(s->d_long_off, 0, sizeof(int32_t), stream));
    }
    const int64_t T = ((int64_t)long_total + LAPIS_TILE_NNZ - 1) / LAPIS_TILE_NNZ;
    s->num_tiles = T;
    if (int rc = device_alloc(&s->d_tile_row, sizeof(int32_t) * ((size_t)T + 1))) return rc;
    if (int rc = device_alloc(&s->d_tile_nz, sizeof(int32_t) * ((size_t)T + 1))) return rc;
    if (int rc = device_alloc(&s->d_partial, esize * 2 * (size_t)T)) return rc;
    tile_search_kernel<LAPIS_TILE_NNZ><<<dim3((uint32_t)((T + 1 + kBlock - 1) / kBlock)), dim3(kBlock), 0, stream>>>(
        m, T, s->d_long_off, s->d_tile_row, s->d_tile_nz);
    LAPIS_HIP(hipGetLastError());
    LAPIS_HIP(hipStreamSynchronize(stream));
    return LAPIS_OK;
}

// Number of column blocks and their width for the split (0: x is too small to bother).
void split_geometry(int64_t ncols, size_t esize, int64_t *num_blocks, int64_t *width)
{
    const int64_t target = (int64_t)LAPIS_SPLIT_BLOCK_BYTES / (int64_t)esize;
    int64_t nb = (ncols + target - 1) / target;
    if (nb > LAPIS_SPLIT_MAX_BLOCKS) nb = LAPIS_SPLIT_MAX_BLOCKS;
    if (nb < 2) { *num_blocks = 0; *width = 0; return; }
    *num_blocks = nb;
    *width = (ncols + nb - 1) / nb;
}

int run_analysis(lapis_csr *A, hipStream_t stream)
{
    const int64_t n = A->nrows;
    const size_t esize = value_size(A);
    DeviceTemp flags_mem;
    if (int rc = flags_mem.alloc(kNumCheckFlags * sizeof(int32_t))) return rc;
    int32_t *d_flags = flags_mem.as<int32_t>();
    LAPIS_HIP(hipMemsetAsync(d_flags, 0, kNumCheckFlags * sizeof(int32_t), stream));

    // structural checks the kernels rely on (rowptr ends, monotone rowptr, column range), the half
    // bandwidth and whether every row's columns ascend: one pass
    bool rows_sorted = false;
    if (n > 0) {
        int64_t vblocks = ((n > A->nnz ? n : A->nnz) + kCheckTile - 1) / kCheckTile;
        if (vblocks > 2048) vblocks = 2048;          // 8 per CU; each ends with one atomic on the same word
        const int64_t check_tiles = (A->nnz + kCheckTile - 1) / kCheckTile;
        DeviceTemp tile_first;
        if (int rc = tile_first.alloc(sizeof(int32_t) * ((size_t)check_tiles + 1))) return rc;
        check_tile_rows_kernel<<<dim3((uint32_t)((check_tiles + 1 + kBlock - 1) / kBlock)), dim3(kBlock), 0, stream>>>(
            (int32_t)n, check_tiles, A->rowptr, tile_first.as<int32_t>());
        structure_check_kernel<<<dim3((uint32_t)vblocks), dim3(kBlock), 0, stream>>>(
            (int32_t)n, A->ncols, (int32_t)A->nnz, A->rowptr, A->colidx, tile_first.as<int32_t>(), d_flags);
        LAPIS_HIP(hipGetLastError());
        int32_t flags[kNumCheckFlags] = {0};
        if (int rc = read_back(flags, d_flags, sizeof(flags), stream)) return rc;
        if (flags[4]) return fail(LAPIS_ERR_INVALID_ARG, "rowptr[0] must be 0 and rowptr[nrows] must equal nnz");
        if (flags[0]) return fail(LAPIS_ERR_INVALID_ARG, "rowptr is not non-decreasing");
        if (flags[1]) return fail(LAPIS_ERR_INVALID_ARG, "a column index is outside [0, ncols)");
        A->half_bandwidth = flags[2];
        rows_sorted = !flags[3];
        // entries whose successor in the row is the next column: below a quarter of the entries the
        // gathers of a chunk mostly touch a cache line each
        A->scattered_columns = A->nnz > 0 && 4 * (int64_t)flags[5] < A->nnz;
    } else if (A->nnz != 0) {
        return fail(LAPIS_ERR_INVALID_ARG, "nnz must be 0 when nrows is 0");
    }

    // level 1: stream chunks (16-byte loads need 16-byte aligned arrays; otherwise no chunk qualifies)
    const int32_t num_chunks = (int32_t)((n + LAPIS_STREAM_ROWS - 1) / LAPIS_STREAM_ROWS);
    A->num_chunks = num_chunks;
    const bool aligned = reinterpret_cast<uintptr_t>(A->colidx) % 16 == 0 &&
                         reinterpret_cast<uintptr_t>(A->vals) % 16 == 0;
    const int32_t min_nnz = aligned ? LAPIS_STREAM_MIN_NNZ : INT32_MAX;
    DeviceTemp chunk_flag;
    if (int rc = chunk_flag.alloc(sizeof(int32_t) * (size_t)num_chunks)) return rc;
    if (int rc = device_alloc(&A->d_stream_chunks, sizeof(int32_t) * (size_t)num_chunks)) return rc;
    int32_t num_stream = 0;
    bool index16 = false;
    struct NarrowCounts {
        unsigned long long entries[4 + 2 * kStreamClasses];   // in narrow, framed, patterned chunks; pool size;
                                                              // then the last two per class
        int32_t chunks[4 * kStreamClasses]; // per class: narrow, framed, patterned, any of the three
    } h_counts = {};
    bool patterns = false;
    if (n > 0) {
        chunk_flag_kernel<<<dim3((uint32_t)((num_chunks + kBlock - 1) / kBlock)), dim3(kBlock), 0, stream>>>(
            (int32_t)n, num_chunks, LAPIS_STREAM_ROWS, min_nnz, A->rowptr, chunk_flag.as<int32_t>());

        // level 1b: 16-bit column codes for the stream chunks that are narrow or framed, kept only if
        // those chunks hold at least half of the entries
        DeviceTemp narrow;
        if (int rc = narrow.alloc(sizeof(NarrowCounts))) return rc;
        NarrowCounts *d_counts = narrow.as<NarrowCounts>();
        if (int rc = device_alloc(&A->d_chunk_base, sizeof(int32_t) * (size_t)num_chunks)) return rc;
        if (int rc = device_alloc(&A->d_frame_table, sizeof(int32_t) * (size_t)num_chunks * kFrameSlots)) return rc;
        LAPIS_HIP(hipMemsetAsync(A->d_frame_table, 0, sizeof(int32_t) * (size_t)num_chunks * kFrameSlots, stream));
        const uint32_t wblocks = (uint32_t)((num_chunks + kWavesPerBlock - 1) / kWavesPerBlock);
        chunk_span_kernel<<<dim3(wblocks), dim3(kBlock), 0, stream>>>(
            (int32_t)n, num_chunks, LAPIS_STREAM_ROWS, chunk_flag.as<int32_t>(), A->rowptr, A->colidx,
            A->d_chunk_base);
        chunk_frames_kernel<<<dim3(wblocks), dim3(kBlock), 0, stream>>>(
            (int32_t)n, num_chunks, LAPIS_STREAM_ROWS, chunk_flag.as<int32_t>(), A->rowptr, A->colidx,
            A->d_chunk_base, A->d_frame_table);
        // when x is far larger than an L2 (the column split's own condition), a chunk with rows above
        // 64 entries whose columns are neither narrow nor framed is better off in the bins, where
        // the column split orders its gathers: it stops being a stream chunk
        int64_t nb0 = 0, W0 = 0;
        split_geometry(A->ncols, esize, &nb0, &W0);
        if (nb0 > 0)
            chunk_demote_kernel<<<dim3((uint32_t)((num_chunks + kBlock - 1) / kBlock)), dim3(kBlock), 0, stream>>>(
                (int32_t)n, num_chunks, LAPIS_STREAM_ROWS, LAPIS_WAVE, A->rowptr, A->d_chunk_base, chunk_flag.as<int32_t>());
        // level 1c: row patterns of the chunks that still stream
        static_assert(LAPIS_STREAM_ROWS <= kWave && LAPIS_PATTERN_MAX_ROW == kPatternMaxRow &&
                      LAPIS_PATTERN_SLOTS == kPatternSlots && LAPIS_PATTERN_TABLE == kPatternTableSize &&
                      kPatternTableSize == kPatternTable, "pattern limits of the header, the analysis and the kernels");
        DeviceTemp pat_len;
        if (int rc = pat_len.alloc(sizeof(int32_t) * (size_t)num_chunks)) return rc;
        if (int rc = device_alloc(&A->d_row_pat, sizeof(uint16_t) * (size_t)n)) return rc;
        chunk_patterns_kernel<<<dim3(wblocks), dim3(kBlock), 0, stream>>>(
            (int32_t)n, num_chunks, LAPIS_STREAM_ROWS, chunk_flag.as<int32_t>(), A->rowptr, A->colidx,
            pat_len.as<int32_t>(), A->d_row_pat);
        LAPIS_HIP(hipMemsetAsync(d_counts, 0, sizeof(NarrowCounts), stream));
        const uint32_t count_blocks = (uint32_t)((num_chunks + 4 * kCompactBlock - 1) / (4 * kCompactBlock));
        narrow_count_kernel<<<dim3(count_blocks < 256 ? count_blocks : 256), dim3(kCompactBlock), 0, stream>>>(
            (int32_t)n, num_chunks, LAPIS_STREAM_ROWS, chunk_flag.as<int32_t>(), A->rowptr, A->d_chunk_base,
            pat_len.as<int32_t>(), d_counts->entries, d_counts->chunks);
        static_assert(kChunkClasses == kStreamClasses, "one list per stream class");
        DeviceTemp offsets;
        if (int rc = offsets.alloc(sizeof(int32_t) * (kStreamClasses + 1))) return rc;
        const int32_t compact_blocks = (num_chunks + kCompactBlock - 1) / kCompactBlock;
        DeviceTemp class_hist;
        if (int rc = class_hist.alloc(sizeof(int32_t) * (size_t)compact_blocks * kChunkClasses)) return rc;
        chunk_class_hist_kernel<<<dim3((uint32_t)compact_blocks), dim3(kCompactBlock), 0, stream>>>(
            num_chunks, chunk_flag.as<int32_t>(), class_hist.as<int32_t>());
        chunk_class_scan_kernel<<<dim3(1), dim3(kCompactBlock), 0, stream>>>(compact_blocks, class_hist.as<int32_t>(),
                                                                             offsets.as<int32_t>());
        chunk_compact_kernel<<<dim3((uint32_t)compact_blocks), dim3(kCompactBlock), 0, stream>>>(
            num_chunks, chunk_flag.as<int32_t>(), class_hist.as<int32_t>(), A->d_stream_chunks);
        LAPIS_HIP(hipGetLastError());
        if (int rc = read_back(A->h_stream_offset, offsets.as<int32_t>(), sizeof(int32_t) * (kStreamClasses + 1), stream)) return rc;
        num_stream = A->h_stream_offset[kStreamClasses];
        if (int rc = read_back(&h_counts, narrow.p, sizeof(h_counts), stream)) return rc;
        const unsigned long long coded = h_counts.entries[0] + h_counts.entries[1];
        A->narrow_entries = (int64_t)h_counts.entries[0];
        A->framed_entries = (int64_t)h_counts.entries[1];
        index16 = coded > 0 && 2 * coded >= (unsigned long long)A->nnz;
        A->pattern_entries = (int64_t)h_counts.entries[2];
        A->pattern_pool = (int64_t)h_counts.entries[3];
        patterns = h_counts.entries[2] > 0 && 2 * h_counts.entries[2] >= (unsigned long long)A->nnz;
        if (patterns) {
            const int32_t scan_tiles = (int32_t)((num_chunks + kScanTile - 1) / kScanTile);
            DeviceTemp tile_sums;
            if (int rc = tile_sums.alloc(sizeof(int32_t) * ((size_t)scan_tiles + 1))) return rc;
            if (int rc = device_alloc(&A->d_pat_off, sizeof(int32_t) * ((size_t)num_chunks + 1))) return rc;
            if (int rc = device_alloc(&A->d_pat_pool, sizeof(int32_t) * (size_t)A->pattern_pool)) return rc;
            scan_tile_sums_kernel<<<dim3(scan_tiles), dim3(kBlock), 0, stream>>>(num_chunks, pat_len.as<int32_t>(),
                                                                                 tile_sums.as<int32_t>());
            scan_tile_offsets_kernel<<<dim3(1), dim3(kBlock), 0, stream>>>(scan_tiles, tile_sums.as<int32_t>());
            scan_apply_kernel<<<dim3(scan_tiles), dim3(kBlock), 0, stream>>>(num_chunks, pat_len.as<int32_t>(),
                                                                             tile_sums.as<int32_t>(), scan_tiles, A->d_pat_off);
            pattern_pool_kernel<<<dim3(wblocks), dim3(kBlock), 0, stream>>>(
                (int32_t)n, num_chunks, LAPIS_STREAM_ROWS, A->rowptr, A->colidx, A->d_pat_off, A->d_row_pat, A->d_pat_pool);
            LAPIS_HIP(hipGetLastError());
            // SpMM: which stream chunks share rows of X between neighbouring rows; two lists
            if (num_stream > 0) {
                DeviceTemp share_offsets;
                if (int rc = device_alloc(&A->d_share_flag, sizeof(int32_t) * (size_t)num_chunks)) return rc;
                if (int rc = share_offsets.alloc(sizeof(int32_t) * (kChunkClasses + 1))) return rc;
                if (int rc = device_alloc(&A->d_spmm_chunks, sizeof(int32_t) * (size_t)num_stream)) return rc;
                spmm_share_flag_kernel<<<dim3(wblocks), dim3(kBlock), 0, stream>>>(
                    (int32_t)n, num_chunks, chunk_flag.as<int32_t>(), A->rowptr,
                    StreamPatterns{A->d_pat_off, A->d_row_pat, A->d_pat_pool}, A->d_share_flag);
                chunk_class_hist_kernel<<<dim3((uint32_t)compact_blocks), dim3(kCompactBlock), 0, stream>>>(
                    num_chunks, A->d_share_flag, class_hist.as<int32_t>());
                chunk_class_scan_kernel<<<dim3(1), dim3(kCompactBlock), 0, stream>>>(compact_blocks, class_hist.as<int32_t>(),
                                                                                     share_offsets.as<int32_t>());
                chunk_compact_kernel<<<dim3((uint32_t)compact_blocks), dim3(kCompactBlock), 0, stream>>>(
                    num_chunks, A->d_share_flag, class_hist.as<int32_t>(), A->d_spmm_chunks);
                LAPIS_HIP(hipGetLastError());
                static_assert(kSharePlain == 1 && kShareNone == 2 && kShareBlock3 == 3 && kShareBlock2 == 4 && kChunkClasses == 4,
                              "the share classes are the four classes of the compaction");
                static_assert(kSharePlain == LAPIS_SHARE_PLAIN && kShareNone == LAPIS_SHARE_NONE && kShareBlock3 == LAPIS_SHARE_BLOCK3 &&
                              kShareBlock2 == LAPIS_SHARE_BLOCK2 && kShareMaxOdd == LAPIS_SHARE_MAX_ODD, "as the header says");
                if (int rc = read_back(A->h_spmm_offset, share_offsets.p, sizeof(A->h_spmm_offset), stream)) return rc;
                if (A->h_spmm_offset[kShareNone] - A->h_spmm_offset[kShareNone - 1] == num_stream) {   // nothing shares
                    (void)hipFree(A->d_spmm_chunks);
                    A->d_spmm_chunks = nullptr;
                }
            }
            LAPIS_HIP(hipStreamSynchronize(stream));       // pat_len and tile_sums are released on return
            for (int cls = 1; cls <= kStreamClasses; ++cls) {
                const int32_t size = A->h_stream_offset[cls] - A->h_stream_offset[cls - 1];
                // each of the class's 2^(cls-1) wavefronts per chunk loads the chunk's whole table (4
                // bytes a diagonal) instead of its share of 2-byte codes: worth it while that is at most
                // half as much
                const unsigned long long waves = 1ull << (cls - 1);
                const bool pays = 4 * waves * h_counts.entries[4 + kStreamClasses + cls - 1] <= h_counts.entries[4 + cls - 1];
                A->class_allpattern[cls - 1] = pays && h_counts.chunks[2 * kStreamClasses + cls - 1] == size;
                A->class_pattern16[cls - 1] = pays && index16 && h_counts.chunks[2 * kStreamClasses + cls - 1] > 0 &&
                                              h_counts.chunks[3 * kStreamClasses + cls - 1] == size;
            }
        }
        if (index16) {
            const size_t len = ((size_t)A->nnz + 7) / 8 * 8 + 8;      // 16-byte loads may run past nnz
            if (int rc = device_alloc(&A->d_col16, sizeof(uint16_t) * len)) return rc;
            LAPIS_HIP(hipMemsetAsync(A->d_col16, 0, sizeof(uint16_t) * len, stream));
            col16_fill_kernel<<<dim3(wblocks), dim3(kBlock), 0, stream>>>(
                (int32_t)n, num_chunks, LAPIS_STREAM_ROWS, A->rowptr, A->colidx, A->d_chunk_base, A->d_frame_table,
                A->d_col16);
            LAPIS_HIP(hipGetLastError());
            for (int cls = 1; cls <= kStreamClasses; ++cls) {
                const int32_t size = A->h_stream_offset[cls] - A->h_stream_offset[cls - 1];
                A->class_all16[cls - 1] = h_counts.chunks[cls - 1] == size;
                A->class_allframed[cls - 1] = h_counts.chunks[kStreamClasses + cls - 1] == size;
                A->class_allcoded[cls - 1] = h_counts.chunks[cls - 1] + h_counts.chunks[kStreamClasses + cls - 1] == size;
            }
        }
    }
    A->num_stream = num_stream;
    if (!patterns) {
        (void)hipFree(A->d_row_pat);
        A->d_row_pat = nullptr;
    }
    if (!index16) {
        (void)hipFree(A->d_chunk_base);
        (void)hipFree(A->d_frame_table);
        A->d_chunk_base = nullptr;
        A->d_frame_table = nullptr;
    }

    // level 2: bins over the remaining rows
    A->rows.num_rows = n;
    A->rows.row_begin = A->rowptr;
    A->rows.row_end = A->rowptr + 1;
    if (int rc = bin_row_set(&A->rows, chunk_flag.as<int32_t>(), esize, stream)) return rc;

    // column split of the rows of the last two bins: rows above LAPIS_HUGE_ROW entries are cut at
    // LDS-sized column blocks, the others at the coarse blocks into virtual rows
    int64_t nb = 0, W = 0;
    split_geometry(A->ncols, esize, &nb, &W);
    const int64_t R89 = A->rows.h_bin_offset[kNumBins] - A->rows.h_bin_offset[kNumBins - 2];
    const int64_t fW = (int64_t)LAPIS_LDS_BLOCK_BYTES / (int64_t)esize;
    const int64_t nbf = (A->ncols + fW - 1) / fW;
    bool split = nb > 0 && R89 > 0;
    const int32_t *rows89 = A->rows.d_row_perm + A->rows.h_bin_offset[kNumBins - 2];
    if (split && !rows_sorted) {   // some row is unsorted: look at these rows themselves
        LAPIS_HIP(hipMemsetAsync(d_flags, 0, sizeof(int32_t), stream));
        const uint32_t sblocks = (uint32_t)(R89 < 65536 ? R89 : 65536);
        split_sorted_kernel<<<dim3(sblocks), dim3(kBlock), 0, stream>>>((int32_t)R89, rows89, A->rowptr,
                                                                        A->colidx, d_flags);
        int32_t unsorted = 0;
        if (int rc = read_back(&unsorted, d_flags, sizeof(int32_t), stream)) return rc;
        split = !unsorted;
    }
    int64_t S = 0, H = 0;
    if (split) {
        if (int rc = device_alloc(&A->d_split_rows, sizeof(int32_t) * (size_t)R89)) return rc;
        if (int rc = device_alloc(&A->d_huge_rows, sizeof(int32_t) * (size_t)R89)) return rc;
        split_rows_kernel<<<dim3(1), dim3(kCompactBlock), 0, stream>>>(
            (int32_t)R89, LAPIS_HUGE_ROW, rows89, A->rowptr, A->d_split_rows, A->d_huge_rows, d_flags);
        LAPIS_HIP(hipGetLastError());
        int32_t counts[2] = {0, 0};
        if (int rc = read_back(counts, d_flags, sizeof(counts), stream)) return rc;
        S = counts[0];
        H = counts[1];
        split = (nb + 1) * S <= INT32_MAX && (nbf + 1) * H <= INT32_MAX;
    }
    if (split) {
        const int64_t cuts = (nb + 1) * S;
        if (int rc = device_alloc(&A->d_cut, sizeof(int32_t) * (size_t)cuts)) return rc;
        if (int rc = device_alloc(&A->d_vsum, esize * (size_t)(nb * S))) return rc;
        if (S > 0)
            split_cut_kernel<<<dim3((uint32_t)((cuts + kBlock - 1) / kBlock)), dim3(kBlock), 0, stream>>>(
                (int32_t)S, (int32_t)nb, W, A->d_split_rows, A->rowptr, A->colidx, A->d_cut);
        LAPIS_HIP(hipGetLastError());
        A->num_blocks = nb;
        A->block_width = W;
        A->num_split = S;
        A->vrows.num_rows = nb * S;
        A->vrows.row_begin = A->d_cut;
        A->vrows.row_end = A->d_cut + S;
        if (int rc = bin_row_set(&A->vrows, nullptr, esize, stream)) return rc;
        const int64_t fcuts = (nbf + 1) * H;
        if (int rc = device_alloc(&A->d_fcut, sizeof(int32_t) * (size_t)fcuts)) return rc;
        if (int rc = device_alloc(&A->d_fsum, esize * (size_t)(nbf * H))) return rc;
        if (H > 0)
            split_cut_kernel<<<dim3((uint32_t)((fcuts + kBlock - 1) / kBlock)), dim3(kBlock), 0, stream>>>(
                (int32_t)H, (int32_t)nbf, fW, A->d_huge_rows, A->rowptr, A->colidx, A->d_fcut);
        LAPIS_HIP(hipGetLastError());
        A->num_huge = H;
        A->num_fblocks = nbf;
        A->fblock_width = fW;
        LAPIS_HIP(hipStreamSynchronize(stream));
    }
    build_short_plan(A->rows, split ? kNumBins - 3 : kShortBins - 1, &A->plan_rows);
    if (split) build_short_plan(A->vrows, kShortBins - 1, &A->plan_vrows);
    if (split || A->rows.num_long > 0) LAPIS_HIP(hipEventCreateWithFlags(&A->scratch_event, hipEventDisableTiming));
    return LAPIS_OK;
}

// CSR arrays of A^T into B->own_* (B's sizes are set): count, scan, fill, sort, gather.
int build_transposed_arrays(const lapis_csr *A, lapis_csr *B, hipStream_t stream)
{
    const int64_t nt = B->nrows, nnz = A->nnz;      // rows of A^T = columns of A
    const size_t esize = value_size(A);
    if (int rc = device_alloc(&B->own_rowptr, sizeof(int32_t) * (size_t)(nt + 1))) return rc;
    if (int rc = device_alloc(&B->own_colidx, sizeof(int32_t) * (size_t)nnz)) return rc;
    {
        char *v = nullptr;
        if (int rc = device_alloc(&v, esize * (size_t)nnz)) return rc;
        B->own_vals = v;
    }
    if (nnz == 0) {
        LAPIS_HIP(hipMemsetAsync(B->own_rowptr, 0, sizeof(int32_t) * (size_t)(nt + 1), stream));
        LAPIS_HIP(hipStreamSynchronize(stream));
        return LAPIS_OK;
    }
    // stable radix sort of (column, entry id) by column, 8 bits per pass
    int bits = 1;
    while (bits < 31 && ((int64_t)1 << bits) < nt) ++bits;
    const int passes = (bits + kRadixBits - 1) / kRadixBits;
    const int32_t num_waves = (int32_t)((nnz + kRadixPerWave - 1) / kRadixPerWave);
    const int64_t counts = (int64_t)kRadixDigits * num_waves;
    const int32_t scan_tiles = (int32_t)((counts + kScanTile - 1) / kScanTile);
    const int64_t check_tiles = (nnz + kCheckTile - 1) / kCheckTile;
    // two pairs of buffers take turns; the arrays of A^T itself serve as the second pair (they
    // are written last, from the first pair, which therefore has to hold the last pass's output)
    DeviceTemp keys_t, vals_t, count, offset, tile_sums, entry_row, tile_first;
    if (int rc = keys_t.alloc(sizeof(int32_t) * (size_t)nnz)) return rc;
    if (int rc = vals_t.alloc(sizeof(int32_t) * (size_t)nnz)) return rc;
    int32_t *const keys_pair[2] = {keys_t.as<int32_t>(), static_cast<int32_t *>(B->own_vals)};
    int32_t *const vals_pair[2] = {vals_t.as<int32_t>(), B->own_colidx};
    if (int rc = count.alloc(sizeof(int32_t) * (size_t)counts)) return rc;
    if (int rc = offset.alloc(sizeof(int32_t) * ((size_t)counts + 1))) return rc;
    if (int rc = tile_sums.alloc(sizeof(int32_t) * ((size_t)scan_tiles + 1))) return rc;
    if (int rc = entry_row.alloc(sizeof(int32_t) * (size_t)nnz)) return rc;
    if (int rc = tile_first.alloc(sizeof(int32_t) * ((size_t)check_tiles + 1))) return rc;
    const uint32_t wave_blocks = (uint32_t)((num_waves + kWavesPerBlock - 1) / kWavesPerBlock);
    const int32_t *keys_in = A->colidx, *vals_in = nullptr;
    for (int pass = 0; pass < passes; ++pass) {
        const int shift = pass * kRadixBits;
        const int to = (passes - 1 - pass) % 2;         // the last pass writes pair 0
        int32_t *keys_out = keys_pair[to], *vals_out = vals_pair[to];
        radix_count_kernel<<<dim3(wave_blocks), dim3(kBlock), 0, stream>>>((int32_t)nnz, num_waves, shift, keys_in,
                                                                          count.as<int32_t>());
        scan_tile_sums_kernel<<<dim3(scan_tiles), dim3(kBlock), 0, stream>>>(counts, count.as<int32_t>(),
                                                                             tile_sums.as<int32_t>());
        scan_tile_offsets_kernel<<<dim3(1), dim3(kBlock), 0, stream>>>(scan_tiles, tile_sums.as<int32_t>());
        scan_apply_kernel<<<dim3(scan_tiles), dim3(kBlock), 0, stream>>>(counts, count.as<int32_t>(), tile_sums.as<int32_t>(),
                                                                         scan_tiles, offset.as<int32_t>());
        radix_scatter_kernel<<<dim3(wave_blocks), dim3(kBlock), 0, stream>>>(
            (int32_t)nnz, num_waves, shift, keys_in, vals_in, offset.as<int32_t>(), keys_out, vals_out);
        keys_in = keys_out;
        vals_in = vals_out;
    }
    int64_t pblocks = (nnz + 1 + kBlock - 1) / kBlock;
    if (pblocks > 65536) pblocks = 65536;
    sorted_keys_to_ptr_kernel<<<dim3((uint32_t)pblocks), dim3(kBlock), 0, stream>>>((int32_t)nnz, (int32_t)nt, keys_in,
                                                                                    B->own_rowptr);
    // the row of every entry of A, then rows and values in sorted order
    check_tile_rows_kernel<<<dim3((uint32_t)((check_tiles + 1 + kBlock - 1) / kBlock)), dim3(kBlock), 0, stream>>>(
        (int32_t)A->nrows, check_tiles, A->rowptr, tile_first.as<int32_t>());
    int64_t rblocks = check_tiles < 8192 ? check_tiles : 8192;
    entry_rows_kernel<<<dim3((uint32_t)rblocks), dim3(kBlock), 0, stream>>>((int32_t)nnz, A->rowptr, tile_first.as<int32_t>(),
                                                                            entry_row.as<int32_t>());
    int64_t gblocks = (nnz + kBlock - 1) / kBlock;
    if (gblocks > 65536) gblocks = 65536;
    if (A->dtype == LAPIS_F64)
        transpose_gather_sorted_kernel<double><<<dim3((uint32_t)gblocks), dim3(kBlock), 0, stream>>>(
            (int32_t)nnz, vals_in, entry_row.as<int32_t>(), static_cast<const double *>(A->vals), B->own_colidx,
            static_cast<double *>(B->own_vals));
    else
        transpose_gather_sorted_kernel<float><<<dim3((uint32_t)gblocks), dim3(kBlock), 0, stream>>>(
            (int32_t)nnz, vals_in, entry_row.as<int32_t>(), static_cast<const float *>(A->vals), B->own_colidx,
            static_cast<float *>(B->own_vals));
    LAPIS_HIP(hipGetLastError());
    LAPIS_HIP(hipStreamSynchronize(stream));     // the temporaries are freed on return
    return LAPIS_OK;
}

// Short-row and long-row kernels over one binned set; results go to out[row id of the set].
template <typename T>
void launch_binned(const lapis_csr *A, const BinnedSet &s, const ShortPlan &plan, bool with_long, const T *x,
                   T *out, T a, T b, T *partial, hipStream_t stream)
{
    const T *vals = static_cast<const T *>(A->vals);
    if (plan.num_blocks > 0) {
        spmv_short_kernel<T, true><<<dim3(plan.num_blocks), dim3(kBlock), 0, stream>>>(
            plan, s.d_row_perm, s.row_begin, s.row_end, A->colidx, vals, x, out, a, b);
    }
    if (with_long && s.num_long > 0) {
        const int32_t m = (int32_t)s.num_long;
        const int32_t *long_rows = s.d_row_perm + s.h_bin_offset[kNumBins - 1];
        spmv_long_tile_kernel<T, LAPIS_TILE_NNZ><<<dim3((uint32_t)s.num_tiles), dim3(kBlock), 0, stream>>>(
            m, long_rows, s.d_long_off, s.d_tile_row, s.d_tile_nz, s.row_begin, A->colidx, vals, x, partial);
        spmv_long_fixup_kernel<T, LAPIS_TILE_NNZ><<<dim3((uint32_t)((m + kWavesPerBlock - 1) / kWavesPerBlock)), dim3(kBlock), 0, stream>>>(
            m, long_rows, s.d_long_off, s.d_tile_row, partial, out, a, b);
    }
}

// Which instantiation of the stream kernel serves the chunks of the classes lo..hi when they are launched
// together with G lanes per row: decided by what ALL their chunks have (empty classes do not count).
enum StreamVariant { kVariantGrouped, kVariantPattern, kVariantPatternOr16, kVariantNarrow, kVariantFramed,
                     kVariantEither, kVariant32 };
StreamVariant stream_variant(const lapis_csr *A, int lo, int hi, int G)
{
    bool all16 = true, allframed = true, allcoded = true, allpattern = true, pattern16 = true;
    for (int cls = lo; cls <= hi; ++cls) {
        if (A->h_stream_offset[cls] == A->h_stream_offset[cls - 1]) continue;
        all16 = all16 && A->class_all16[cls - 1];
        allframed = allframed && A->class_allframed[cls - 1];
        allcoded = allcoded && A->class_allcoded[cls - 1];
        allpattern = allpattern && A->class_allpattern[cls - 1];
        pattern16 = pattern16 && (A->class_pattern16[cls - 1] || A->class_allpattern[cls - 1]);
    }
    // With scattered columns every gather is a cache line of its own and the time goes into L1
    // misses: the wavefronts of a chunk then run as one workgroup, on one CU, where the lines one
    // of them fetched serve the others (stand-ins 7 and 9: 143 -> 137 us, 309 -> 291 us).  Where
    // columns come in runs the same grouping costs time (Elasticity3D stand-in 94 -> 107 us).
    // Neighbouring one-wavefront chunks (G == 2) gain nothing from it.
    if (A->scattered_columns && all16 && !allpattern && !pattern16 && G >= 4) return kVariantGrouped;
    if (allpattern) return kVariantPattern;
    if (pattern16) return kVariantPatternOr16;
    if (all16) return kVariantNarrow;
    if (allframed) return kVariantFramed;
    if (allcoded) return kVariantEither;
    return kVariant32;
}

// Stream chunks of the classes lo..hi (their lists are neighbours) with the lane groups of class hi,
// G lanes per row: one wavefront per 64/G rows.  A chunk of a lower class meets the limits of every
// higher one (rows and entries per chunk), only with more lanes per row than it needs.
template <typename T, int G>
void launch_stream(const lapis_csr *A, int lo, int hi, const T *x, T *y, T a, T b, hipStream_t stream)
{
    const int64_t count = A->h_stream_offset[hi] - A->h_stream_offset[lo - 1];
    if (count == 0) return;
    const uint32_t waves = (uint32_t)(count * (G / 2));
    const uint32_t padded = (waves + kXcds - 1) / kXcds * kXcds;
    const int32_t *list = (count == A->num_chunks) ? nullptr : A->d_stream_chunks + A->h_stream_offset[lo - 1];
#define LAPIS_STREAM_LAUNCH(RAW)                                                                             \
    spmv_stream_kernel<T, G, true, RAW><<<dim3(padded), dim3(kWave), 0, stream>>>(                            \
        (int32_t)A->nrows, (int32_t)A->nnz, waves, padded, list, A->rowptr, A->colidx, A->d_chunk_base,        \
        A->d_frame_table, A->d_col16, StreamPatterns{A->d_pat_off, A->d_row_pat, A->d_pat_pool},              \
        static_cast<const T *>(A->vals), x, y, a, b)
#define LAPIS_STREAM_GROUPED(GWV)                                                                            \
    do {                                                                                                     \
        const uint32_t groups = (waves + (GWV) - 1) / (GWV), pgroups = (groups + kXcds - 1) / kXcds * kXcds;  \
        spmv_stream_kernel<T, G, true, kColsNarrow, kStreamUnroll, GWV><<<dim3(pgroups), dim3(kWave * (GWV)), 0, stream>>>( \
            (int32_t)A->nrows, (int32_t)A->nnz, waves, pgroups, list, A->rowptr, A->colidx, A->d_chunk_base,   \
            A->d_frame_table, A->d_col16, StreamPatterns{A->d_pat_off, A->d_row_pat, A->d_pat_pool},          \
            static_cast<const T *>(A->vals), x, y, a, b);                                                     \
    } while (0)
    switch (stream_variant(A, lo, hi, G)) {
    case kVariantGrouped:
        if constexpr (G >= 4) LAPIS_STREAM_GROUPED(G / 2);
        break;
    case kVariantPattern: LAPIS_STREAM_LAUNCH(kColsPattern); break;
    case kVariantPatternOr16: LAPIS_STREAM_LAUNCH(kColsPatternOr16); break;
    case kVariantNarrow: LAPIS_STREAM_LAUNCH(kColsNarrow); break;
    case kVariantFramed: LAPIS_STREAM_LAUNCH(kColsFramed); break;
    case kVariantEither: LAPIS_STREAM_LAUNCH(kColsEither); break;
    case kVariant32: LAPIS_STREAM_LAUNCH(kCols32); break;
    }
#undef LAPIS_STREAM_GROUPED
#undef LAPIS_STREAM_LAUNCH
}

template <typename T>
void launch_stream_classes(const lapis_csr *A, int lo, int hi, const T *x, T *y, T a, T b, hipStream_t stream)
{
    switch (hi) {
    case 1: launch_stream<T, 2>(A, lo, hi, x, y, a, b, stream); break;
    case 2: launch_stream<T, 4>(A, lo, hi, x, y, a, b, stream); break;
    case 3: launch_stream<T, 8>(A, lo, hi, x, y, a, b, stream); break;
    default: launch_stream<T, 16>(A, lo, hi, x, y, a, b, stream); break;
    }
}

// All stream chunks.  Kernels of one stream run one after the other, so a class with few chunks costs a
// launch that cannot fill the GPU (7 to 8 us on the Elasticity3D stand-in: the chunks at the grid's
// faces).  Such a class rides with the next class up that has chunks - at most an eighth as many as
// that class has, and only if the kernel variant that class would get by itself still serves both.
template <typename T>
void launch_all_streams(const lapis_csr *A, const T *x, T *y, T a, T b, hipStream_t stream)
{
    const int32_t *off = A->h_stream_offset;
    int lo = 1, top = 0;                       // pending classes lo..top (top = the highest of them with chunks)
    for (int cls = 1; cls <= kStreamClasses; ++cls) {
        const int64_t here = off[cls] - off[cls - 1];
        if (here == 0) continue;
        const int64_t pending = off[cls - 1] - off[lo - 1];
        if (pending > 0) {
            const int G = 1 << cls;
            const bool rides = pending * 8 <= here && stream_variant(A, lo, cls, G) == stream_variant(A, cls, cls, G);
            if (!rides) {
                launch_stream_classes<T>(A, lo, top, x, y, a, b, stream);
                lo = cls;
            }
        } else {
            lo = cls;
        }
        top = cls;
    }
    if (top > 0) launch_stream_classes<T>(A, lo, top, x, y, a, b, stream);
}

// y (ncols values) = beta*y, then every entry of A adds alpha*vals[j]*x[row] into y[colidx[j]].
template <typename T>
int spmv_transpose_typed(const lapis_csr *A, double alpha, const void *d_x, double beta, void *d_y,
                         hipStream_t stream)
{
    T *y = static_cast<T *>(d_y);
    int64_t blocks = (A->ncols + kBlock - 1) / kBlock;
    if (blocks > 16384) blocks = 16384;
    transpose_scale_kernel<T><<<dim3((uint32_t)blocks), dim3(kBlock), 0, stream>>>(A->ncols, y, (T)beta);
    if (A->nnz > 0) {
        const uint32_t tiles = (uint32_t)((A->nnz + kScatterTile - 1) / kScatterTile);
        transpose_scatter_kernel<T><<<dim3(tiles), dim3(kBlock), 0, stream>>>(
            (int32_t)A->nrows, (int32_t)A->nnz, A->rowptr, A->colidx, static_cast<const T *>(A->vals),
            static_cast<const T *>(d_x), y, (T)alpha);
    }
    LAPIS_HIP(hipGetLastError());
    return LAPIS_OK;
}

// Device address of `scratch` on the current device: asked for once per device, with that
// device current, and kept (every GPU holds its own copy of the array at its own address).
int static_scratch_address(unsigned char **out)
{
    constexpr int kMaxDevices = 64;
    static std::mutex lock;
    static unsigned char *address[kMaxDevices] = {nullptr};
    int dev = -1;
    LAPIS_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(LAPIS_ERR_DEVICE, "device ordinal beyond the static scratch table");
    std::lock_guard<std::mutex> guard(lock);
    if (!address[dev]) {
        void *ptr = nullptr;
        LAPIS_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return fail(LAPIS_ERR_DEVICE, "hipGetSymbolAddress returned a null address");
        address[dev] = static_cast<unsigned char *>(ptr);
    }
    *out = address[dev];
    return LAPIS_OK;
}

template <typename T>
const T *vals_of(const lapis_csr *A) { return static_cast<const T *>(A->vals); }

// Where a product keeps its intermediate sums: per-tile sums of the long rows (2 per tile) of the
// matrix's own rows and of the virtual rows, one sum per virtual row, one per (LDS block, huge row).
// Every element that is read has been written earlier in the same call, so nothing needs clearing.
struct SpmvScratch {
    void *partial_rows, *partial_vrows, *vsum, *fsum;
};

SpmvScratch handle_scratch(const lapis_csr *A)
{
    return SpmvScratch{A->rows.d_partial, A->vrows.d_partial, A->d_vsum, A->d_fsum};
}

template <typename T>
int spmv_typed(const lapis_csr *A, double alpha, const void *d_x, double beta, void *d_y, const SpmvScratch &scr,
               hipStream_t stream)
{
    const T a = (T)alpha, b = (T)beta;
    const T *x = static_cast<const T *>(d_x);
    T *y = static_cast<T *>(d_y);
    launch_all_streams<T>(A, x, y, a, b, stream);
    const bool split = A->num_blocks > 0;
    launch_binned<T>(A, A->rows, A->plan_rows, !split, x, y, a, b, static_cast<T *>(scr.partial_rows), stream);
    if (split) {
        // rows above 64 entries: their column-block pieces first, then one sum per row
        T *vsum = static_cast<T *>(scr.vsum);
        launch_binned<T>(A, A->vrows, A->plan_vrows, true, x, vsum, T(1), T(0), static_cast<T *>(scr.partial_vrows), stream);
        if (A->num_split > 0)
            split_combine_kernel<T><<<dim3((uint32_t)((A->num_split + kBlock - 1) / kBlock)), dim3(kBlock), 0, stream>>>(
                (int32_t)A->num_split, (int32_t)A->num_blocks, A->d_split_rows, vsum, y, a, b);
        if (A->num_huge > 0) {
            // rows above LAPIS_HUGE_ROW entries: pieces per LDS-sized block of x, then one sum per row
            T *fsum = static_cast<T *>(scr.fsum);
            const int64_t H = A->num_huge, nbf = A->num_fblocks;
            int64_t groups = (8 * 256 + nbf - 1) / nbf;                      // about 8 workgroups per CU in all
            const int64_t most = (H + kLdsBlockWaves - 1) / kLdsBlockWaves;  // one piece per wavefront at least
            if (groups > most) groups = most;
            if (groups < 1) groups = 1;
            if (groups > 65535) groups = 65535;
            spmv_ldsblock_kernel<T><<<dim3((uint32_t)nbf, (uint32_t)groups), dim3(kLdsBlockThreads),
                                      (size_t)LAPIS_LDS_BLOCK_BYTES, stream>>>(
                (int32_t)H, (int32_t)A->fblock_width, A->ncols, A->d_fcut, A->colidx, vals_of<T>(A), x, fsum);
            spmv_ldsblock_combine_kernel<T><<<dim3((uint32_t)((H + kWavesPerBlock - 1) / kWavesPerBlock)), dim3(kBlock), 0, stream>>>(
                (int32_t)H, (int32_t)nbf, A->d_huge_rows, fsum, y, a, b);
        }
    }
    LAPIS_HIP(hipGetLastError());
    return LAPIS_OK;
}

template <typename T, int G>
void launch_vector(const lapis_csr *A, T a, const T *x, T b, T *y, hipStream_t stream)
{
    const uint32_t blocks = (uint32_t)((A->nrows + (kBlock / G) - 1) / (kBlock / G));
    spmv_vector_kernel<T, G><<<dim3(blocks), dim3(kBlock), 0, stream>>>(
        (int32_t)A->nrows, A->rowptr, A->colidx, static_cast<const T *>(A->vals), x, y, a, b);
}

template <typename T>
int spmv_paper_shape_typed(const lapis_csr *A, double alpha, const void *d_x, double beta, void *d_y,
                           hipStream_t stream)
{
    const int g = lapis_paper_vector_length(A->nrows, A->nnz);
    const T a = (T)alpha, b = (T)beta;
    const T *x = static_cast<const T *>(d_x);
    T *y = static_cast<T *>(d_y);
    switch (g) {
    case 1: launch_vector<T, 1>(A, a, x, b, y, stream); break;
    case 2: launch_vector<T, 2>(A, a, x, b, y, stream); break;
    case 4: launch_vector<T, 4>(A, a, x, b, y, stream); break;
    case 8: launch_vector<T, 8>(A, a, x, b, y, stream); break;
    case 16: launch_vector<T, 16>(A, a, x, b, y, stream); break;
    case 32: launch_vector<T, 32>(A, a, x, b, y, stream); break;
    default: launch_vector<T, 64>(A, a, x, b, y, stream); break;
    }
    LAPIS_HIP(hipGetLastError());
    return LAPIS_OK;
}

// SpMM launches over at most kFewChunks stream chunks of a matrix with kLongRowsMean entries per row or more
// give every pass of a chunk a wavefront of its own
constexpr uint32_t kFewChunks = 8192;
constexpr int64_t kLongRowsMean = 48;

template <typename T, int VEC, int CL>
int spmm_launch(const lapis_csr *A, int64_t k, T a, const T *X, int64_t ldx, T b, T *Y, int64_t ldy,
                hipStream_t stream)
{
    const T *vals = static_cast<const T *>(A->vals);
    const BinnedSet &s = A->rows;
    const int32_t n_rows_a = s.h_bin_offset[kNumBins - 2];            // bins 0..7: one slot per row
    const int32_t n_rows_b = (int32_t)s.num_binned - n_rows_a;        // bins 8..9: one workgroup per row
    constexpr int kSlots = kBlock / CL;
    if (A->num_stream > 0) {                                          // rows of the stream chunks
        const uint32_t chunks = (uint32_t)A->num_stream;
        const int32_t *list = (A->num_stream == A->num_chunks) ? nullptr : A->d_stream_chunks;  // any order
        constexpr int kStreamLanes = CL > 16 ? 16 : CL;               // wider rows of X: several column blocks
        // Rows of X a band-wide window of matrix rows touches: if they overflow an XCD's L2 when one
        // XCD walks the window alone, deal the chunks to the XCDs block-cyclically (block = 1/8 of
        // the half bandwidth) so that the 8 L2s share the window.  Only when every chunk streams
        // (the list is then the identity and chunk order = row order).
        const int64_t cols_here = k < (int64_t)kStreamLanes * VEC ? k : (int64_t)kStreamLanes * VEC;
        const int64_t window_bytes = (2 * A->half_bandwidth + 1) * cols_here * (int64_t)sizeof(T);
        uint32_t xcd_block = 0;
        if (!list && window_bytes > (int64_t)LAPIS_SPLIT_BLOCK_BYTES) {
            const int64_t b = A->half_bandwidth / kXcds / LAPIS_STREAM_ROWS;
            if (b >= 1 && b * kXcds < chunks) xcd_block = (uint32_t)b;
        }
        const uint32_t unit = xcd_block ? xcd_block * kXcds : kXcds;
        const uint32_t padded = (chunks + unit - 1) / unit * unit;
        // every stream chunk has 16-bit offsets, and offset * (bytes per row of X) fits in 32 bits
        bool all16 = A->d_col16 != nullptr && ldx * (int64_t)sizeof(T) <= 0xffff;
        for (int cls = 1; cls <= kStreamClasses; ++cls)
            all16 = all16 && (A->class_all16[cls - 1] || A->h_stream_offset[cls] == A->h_stream_offset[cls - 1]);
        // chunks whose neighbouring rows share rows of X go to the kernel that loads those rows once per
        // R rows (8 or 16 lanes per row of X; a row of X shorter than 16 MiB), by share class; the others follow
        bool share_ok = false;
        if constexpr (kStreamLanes >= 8) share_ok = A->d_spmm_chunks && ldx * (int64_t)sizeof(T) < ((int64_t)1 << 24);
        const StreamPatterns pats{A->d_pat_off, A->d_row_pat, A->d_pat_pool};
        // One share class over columns [c0, ...): when every chunk of the matrix streams and nearly all of them
        // are of this class (all but a few at the ends of the matrix), the kernel is launched over all chunks in
        // the block-cyclic order above and skips the others by their flag: no list to read before the first
        // load, windows of X still shared by the XCDs.  Otherwise over the class's list.
        auto launch_share = [&](auto delta_tag, int32_t cls, int64_t c0) {
            constexpr int DELTA = decltype(delta_tag)::value;
            const uint32_t first = (uint32_t)A->h_spmm_offset[cls - 1], n = (uint32_t)A->h_spmm_offset[cls] - first;
            if (n == 0) return;
            const bool by_flag = !list && (uint64_t)n * 10 >= (uint64_t)chunks * 9;
            const uint32_t count = by_flag ? chunks : n;
            const uint32_t grid = by_flag ? padded : (n + kXcds - 1) / kXcds * kXcds;
            const int32_t *ids = by_flag ? nullptr : A->d_spmm_chunks + first;
            const int32_t *flags = (by_flag && n != chunks) ? A->d_share_flag : nullptr;
            if constexpr (kStreamLanes >= 8) {
                if constexpr (DELTA == 0) {
                    spmm_shared_kernel<T, VEC, kStreamLanes, true><<<dim3(grid), dim3(kWave), 0, stream>>>(
                        (int32_t)A->nrows, (int32_t)A->nnz, count, grid, ids, flags, A->rowptr, by_flag ? xcd_block : 0u,
                        vals, k, c0, X, ldx, Y, ldy, a, b, pats, (int32_t)A->ncols);
                } else {   // block rows: 8 lanes per row of X, so a block of 16 lanes is two launches
                    for (int64_t c1 = c0; c1 < k && c1 < c0 + (int64_t)kStreamLanes * VEC; c1 += 8 * VEC)
                        spmm_block_shared_kernel<T, VEC, true, DELTA, kShareBlockSeg><<<dim3(grid), dim3(kWave), 0, stream>>>(
                            (int32_t)A->nrows, count, grid, ids, flags, cls, A->rowptr, by_flag ? xcd_block : 0u,
                            vals, k, c1, X, ldx, Y, ldy, a, b, pats, (int32_t)A->ncols);
                }
            }
        };
        const uint32_t n_none = share_ok ? (uint32_t)(A->h_spmm_offset[kShareNone] - A->h_spmm_offset[kShareNone - 1]) : chunks;
        const int32_t *none_list = share_ok ? A->d_spmm_chunks + A->h_spmm_offset[kShareNone - 1] : list;
        const uint32_t none_padded = share_ok ? (n_none + kXcds - 1) / kXcds * kXcds : padded;
        const uint32_t none_xcd_block = share_ok ? 0 : xcd_block;
        for (int64_t c0 = 0; c0 < k; c0 += kStreamLanes * VEC) {
            if (share_ok) {
                launch_share(std::integral_constant<int, 0>(), kSharePlain, c0);
                launch_share(std::integral_constant<int, 3>(), kShareBlock3, c0);
                launch_share(std::integral_constant<int, 2>(), kShareBlock2, c0);
            }
            if (n_none == 0) continue;
            // few chunks of long rows (what the share classes left over): a wavefront per pass of a chunk instead
            // of one per chunk, or a dozen wavefronts per CU would each walk their 32 rows alone (Elasticity3D
            // stand-in, 3150 chunks of 81-entry rows: 83 -> 48 us; with 9 entries per row it costs 10 %)
            constexpr uint32_t kParts = kStreamRows / (kWave / kStreamLanes);
            const bool per_pass = kParts > 1 && n_none <= kFewChunks && A->nnz >= kLongRowsMean * A->nrows;
            if (per_pass) {
                const uint32_t units = n_none * kParts, padded_units = (units + kXcds - 1) / kXcds * kXcds;
                if (all16)
                    spmm_stream_kernel<T, VEC, kStreamLanes, true, true, true><<<dim3(padded_units), dim3(kWave), 0, stream>>>(
                        (int32_t)A->nrows, (int32_t)A->nnz, units, padded_units, none_list, A->rowptr, 0u,
                        A->colidx, A->d_chunk_base, A->d_frame_table, A->d_col16, vals, k, c0, X, ldx, Y, ldy, a, b);
                else
                    spmm_stream_kernel<T, VEC, kStreamLanes, true, false, true><<<dim3(padded_units), dim3(kWave), 0, stream>>>(
                        (int32_t)A->nrows, (int32_t)A->nnz, units, padded_units, none_list, A->rowptr, 0u,
                        A->colidx, A->d_chunk_base, A->d_frame_table, A->d_col16, vals, k, c0, X, ldx, Y, ldy, a, b);
            } else if (all16)
                spmm_stream_kernel<T, VEC, kStreamLanes, true, true><<<dim3(none_padded), dim3(kWave), 0, stream>>>(
                    (int32_t)A->nrows, (int32_t)A->nnz, n_none, none_padded, none_list, A->rowptr, none_xcd_block,
                    A->colidx, A->d_chunk_base, A->d_frame_table, A->d_col16, vals, k, c0, X, ldx, Y, ldy, a, b);
            else
                spmm_stream_kernel<T, VEC, kStreamLanes, true, false><<<dim3(none_padded), dim3(kWave), 0, stream>>>(
                    (int32_t)A->nrows, (int32_t)A->nnz, n_none, none_padded, none_list, A->rowptr, none_xcd_block,
                    A->colidx, A->d_chunk_base, A->d_frame_table, A->d_col16, vals, k, c0, X, ldx, Y, ldy, a, b);
        }
    }
    if (n_rows_a > 0) {
        const uint32_t blocks = (uint32_t)(((int64_t)n_rows_a + kSlots - 1) / kSlots);
        const uint32_t padded = (blocks + kXcds - 1) / kXcds * kXcds;
        spmm_rows_kernel<T, VEC, CL, true><<<dim3(padded), dim3(kBlock), 0, stream>>>(
            n_rows_a, blocks, padded, s.d_row_perm, A->rowptr, A->colidx, vals, k, X, ldx, Y, ldy, a, b);
    }
    if (n_rows_b > 0) {
        spmm_block_rows_kernel<T, VEC, CL><<<dim3((uint32_t)n_rows_b), dim3(kBlock), 0, stream>>>(
            n_rows_a, s.d_row_perm, A->rowptr, A->colidx, vals, k, X, ldx, Y, ldy, a, b);
    }
    LAPIS_HIP(hipGetLastError());
    return LAPIS_OK;
}

template <typename T, int VEC>
int spmm_pick_lanes(const lapis_csr *A, int64_t k, T a, const T *X, int64_t ldx, T b, T *Y, int64_t ldy,
                    hipStream_t stream)
{
    const int64_t need = (k + VEC - 1) / VEC;  // lanes wanted to cover a row of X in one pass
    if (need <= 1) return spmm_launch<T, VEC, 1>(A, k, a, X, ldx, b, Y, ldy, stream);
    if (need <= 2) return spmm_launch<T, VEC, 2>(A, k, a, X, ldx, b, Y, ldy, stream);
    if (need <= 4) return spmm_launch<T, VEC, 4>(A, k, a, X, ldx, b, Y, ldy, stream);
    if (need <= 8) return spmm_launch<T, VEC, 8>(A, k, a, X, ldx, b, Y, ldy, stream);
    if (need <= 16) return spmm_launch<T, VEC, 16>(A, k, a, X, ldx, b, Y, ldy, stream);
    if (need <= 32) return spmm_launch<T, VEC, 32>(A, k, a, X, ldx, b, Y, ldy, stream);
    return spmm_launch<T, VEC, 64>(A, k, a, X, ldx, b, Y, ldy, stream);
}

template <typename T>
int spmm_typed(const lapis_csr *A, int64_t k, double alpha, const void *d_X, int64_t ldx, double beta,
               void *d_Y, int64_t ldy, hipStream_t stream)
{
    constexpr int kVec = 16 / sizeof(T);  // elements per 16-byte load
    const T *X = static_cast<const T *>(d_X);
    T *Y = static_cast<T *>(d_Y);
    const bool wide = (k % kVec == 0) && (ldx % kVec == 0) && (ldy % kVec == 0) &&
                      (reinterpret_cast<uintptr_t>(X) % 16 == 0) && (reinterpret_cast<uintptr_t>(Y) % 16 == 0);
    if (wide) return spmm_pick_lanes<T, kVec>(A, k, (T)alpha, X, ldx, (T)beta, Y, ldy, stream);
    return spmm_pick_lanes<T, 1>(A, k, (T)alpha, X, ldx, (T)beta, Y, ldy, stream);
}

int copy_set(const BinnedSet &s, int32_t *h_bin_offset, int32_t *h_row_perm, int32_t *h_long_off,
             int32_t *h_tile_row, int32_t *h_tile_nz)
{
    if (h_bin_offset) std::memcpy(h_bin_offset, s.h_bin_offset, sizeof(s.h_bin_offset));
    if (h_row_perm && s.num_binned > 0)
        LAPIS_HIP(hipMemcpy(h_row_perm, s.d_row_perm, sizeof(int32_t) * (size_t)s.num_binned, hipMemcpyDeviceToHost));
    if (h_long_off)
        LAPIS_HIP(hipMemcpy(h_long_off, s.d_long_off, sizeof(int32_t) * ((size_t)s.num_long + 1), hipMemcpyDeviceToHost));
    if (h_tile_row)
        LAPIS_HIP(hipMemcpy(h_tile_row, s.d_tile_row, sizeof(int32_t) * ((size_t)s.num_tiles + 1), hipMemcpyDeviceToHost));
    if (h_tile_nz)
        LAPIS_HIP(hipMemcpy(h_tile_nz, s.d_tile_nz, sizeof(int32_t) * ((size_t)s.num_tiles + 1), hipMemcpyDeviceToHost));
    return LAPIS_OK;
}

}  // namespace

extern "C" {

int lapis_csr_create_transpose(lapis_csr_t **out, const lapis_csr_t *A, void *hip_stream)
{
    if (!out) return fail(LAPIS_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (!A) return fail(LAPIS_ERR_INVALID_ARG, "handle is NULL");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    lapis_csr *B = new (std::nothrow) lapis_csr();
    if (!B) return fail(LAPIS_ERR_ALLOC, "host allocation failed");
    B->nrows = A->ncols; B->ncols = A->nrows; B->nnz = A->nnz; B->dtype = A->dtype;
    int rc = build_transposed_arrays(A, B, stream);
    if (rc == LAPIS_OK) {
        B->rowptr = B->own_rowptr; B->colidx = B->own_colidx; B->vals = B->own_vals;
        rc = run_analysis(B, stream);
    }
    if (rc) { const std::string why = g_last_error; (void)free_handle(B); return fail(rc, why); }
    *out = B;
    return LAPIS_OK;
}

int lapis_csr_shape(const lapis_csr_t *A, int64_t *nrows, int64_t *ncols, int64_t *nnz, int *dtype)
{
    if (!A) return fail(LAPIS_ERR_INVALID_ARG, "handle is NULL");
    if (nrows) *nrows = A->nrows;
    if (ncols) *ncols = A->ncols;
    if (nnz) *nnz = A->nnz;
    if (dtype) *dtype = A->dtype;
    return LAPIS_OK;
}

int lapis_csr_copy_arrays(const lapis_csr_t *A, int32_t *h_rowptr, int32_t *h_colidx, void *h_vals)
{
    if (!A) return fail(LAPIS_ERR_INVALID_ARG, "handle is NULL");
    LAPIS_HIP(hipDeviceSynchronize());
    if (h_rowptr) LAPIS_HIP(hipMemcpy(h_rowptr, A->rowptr, sizeof(int32_t) * (size_t)(A->nrows + 1), hipMemcpyDeviceToHost));
    if (h_colidx && A->nnz > 0) LAPIS_HIP(hipMemcpy(h_colidx, A->colidx, sizeof(int32_t) * (size_t)A->nnz, hipMemcpyDeviceToHost));
    if (h_vals && A->nnz > 0) LAPIS_HIP(hipMemcpy(h_vals, A->vals, value_size(A) * (size_t)A->nnz, hipMemcpyDeviceToHost));
    return LAPIS_OK;
}

int lapis_csr_create(lapis_csr_t **out, int64_t nrows, int64_t ncols, int64_t nnz, const int32_t *d_rowptr,
                     const int32_t *d_colidx, const void *d_vals, int dtype, void *hip_stream)
{
    if (!out) return fail(LAPIS_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (nrows < 0 || ncols < 0 || nnz < 0) return fail(LAPIS_ERR_INVALID_ARG, "negative size");
    if (nnz > LAPIS_MAX_NNZ || nrows + 1 > INT32_MAX || ncols > INT32_MAX)
        return fail(LAPIS_ERR_INVALID_ARG, "nnz must not exceed 2^31 - 2^16; nrows+1 and ncols must fit in int32");
    if (dtype != LAPIS_F32 && dtype != LAPIS_F64) return fail(LAPIS_ERR_UNSUPPORTED, "dtype must be LAPIS_F32 or LAPIS_F64");
    if (!d_rowptr) return fail(LAPIS_ERR_INVALID_ARG, "d_rowptr is NULL");
    if (nnz > 0 && (!d_colidx || !d_vals)) return fail(LAPIS_ERR_INVALID_ARG, "d_colidx / d_vals is NULL with nnz > 0");
    if (nnz > 0 && (nrows == 0 || ncols == 0)) return fail(LAPIS_ERR_INVALID_ARG, "nnz > 0 in an empty matrix");

    lapis_csr *A = new (std::nothrow) lapis_csr();
    if (!A) return fail(LAPIS_ERR_ALLOC, "host allocation failed");
    A->nrows = nrows; A->ncols = ncols; A->nnz = nnz; A->dtype = dtype;
    A->rowptr = d_rowptr; A->colidx = d_colidx; A->vals = d_vals;
    const int rc = run_analysis(A, static_cast<hipStream_t>(hip_stream));
    if (rc) { const std::string why = g_last_error; (void)free_handle(A); return fail(rc, why); }
    *out = A;
    return LAPIS_OK;
}

int lapis_spmv(const lapis_csr_t *A, double alpha, const void *d_x, double beta, void *d_y, void *hip_stream)
{
    if (!A) return fail(LAPIS_ERR_INVALID_ARG, "handle is NULL");
    if (A->nrows > 0 && !d_y) return fail(LAPIS_ERR_INVALID_ARG, "d_y is NULL");
    if (A->nnz > 0 && !d_x) return fail(LAPIS_ERR_INVALID_ARG, "d_x is NULL");
    if (A->nrows == 0) return LAPIS_OK;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const SpmvScratch scr = handle_scratch(A);
    if (!A->scratch_event)
        return A->dtype == LAPIS_F64 ? spmv_typed<double>(A, alpha, d_x, beta, d_y, scr, stream)
                                     : spmv_typed<float>(A, alpha, d_x, beta, d_y, scr, stream);
    // this handle's products share its scratch: order them across streams (not while a stream is being
    // captured into a graph: there the caller orders the captured products, as the header says)
    hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
    LAPIS_HIP(hipStreamIsCapturing(stream, &capturing));
    std::lock_guard<std::mutex> guard(A->scratch_lock);
    const bool ordered = capturing == hipStreamCaptureStatusNone;
    if (ordered && A->scratch_used && A->scratch_stream != stream)
        LAPIS_HIP(hipStreamWaitEvent(stream, A->scratch_event, 0));
    const int rc = A->dtype == LAPIS_F64 ? spmv_typed<double>(A, alpha, d_x, beta, d_y, scr, stream)
                                         : spmv_typed<float>(A, alpha, d_x, beta, d_y, scr, stream);
    if (rc != LAPIS_OK) return rc;
    if (ordered) {
        LAPIS_HIP(hipEventRecord(A->scratch_event, stream));
        A->scratch_stream = stream;
        A->scratch_used = true;
    }
    return LAPIS_OK;
}

int64_t lapis_spmv_scratch_bytes(const lapis_csr_t *A)
{
    if (!A) return -1;
    const int64_t e = (int64_t)value_size(A);
    auto up = [](int64_t b) { return (b + 255) / 256 * 256; };
    return up(e * 2 * A->rows.num_tiles) + up(e * 2 * A->vrows.num_tiles) + up(e * A->num_blocks * A->num_split) +
           up(e * A->num_fblocks * A->num_huge);
}

int lapis_spmv_static_scratch(const lapis_csr_t *A, double alpha, const void *d_x, double beta, void *d_y,
                              void *hip_stream)
{
    if (!A) return fail(LAPIS_ERR_INVALID_ARG, "handle is NULL");
    if (A->nrows > 0 && !d_y) return fail(LAPIS_ERR_INVALID_ARG, "d_y is NULL");
    if (A->nnz > 0 && !d_x) return fail(LAPIS_ERR_INVALID_ARG, "d_x is NULL");
    const int64_t need = lapis_spmv_scratch_bytes(A);
    if (need > (int64_t)LAPIS_STATIC_SCRATCH_BYTES)
        return fail(LAPIS_ERR_INVALID_ARG, "lapis_spmv_static_scratch: this matrix needs " + std::to_string(need) +
                                               " bytes of scratch, the static buffer holds " +
                                               std::to_string((int64_t)LAPIS_STATIC_SCRATCH_BYTES) + "; use lapis_spmv");
    if (A->nrows == 0) return LAPIS_OK;
    unsigned char *base = nullptr;
    if (int rc = static_scratch_address(&base)) return rc;
    // the four pieces back to back, each starting at a multiple of 256 bytes
    const int64_t e = (int64_t)value_size(A);
    auto up = [](int64_t b) { return (b + 255) / 256 * 256; };
    SpmvScratch scr;
    scr.partial_rows = base;
    scr.partial_vrows = base + up(e * 2 * A->rows.num_tiles);
    scr.vsum = static_cast<unsigned char *>(scr.partial_vrows) + up(e * 2 * A->vrows.num_tiles);
    scr.fsum = static_cast<unsigned char *>(scr.vsum) + up(e * A->num_blocks * A->num_split);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    return A->dtype == LAPIS_F64 ? spmv_typed<double>(A, alpha, d_x, beta, d_y, scr, stream)
                                 : spmv_typed<float>(A, alpha, d_x, beta, d_y, scr, stream);
}

int lapis_spmv_transpose(const lapis_csr_t *A, double alpha, const void *d_x, double beta, void *d_y,
                         void *hip_stream)
{
    if (!A) return fail(LAPIS_ERR_INVALID_ARG, "handle is NULL");
    if (A->ncols > 0 && !d_y) return fail(LAPIS_ERR_INVALID_ARG, "d_y is NULL");
    if (A->nnz > 0 && !d_x) return fail(LAPIS_ERR_INVALID_ARG, "d_x is NULL");
    if (A->ncols == 0) return LAPIS_OK;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    return A->dtype == LAPIS_F64 ? spmv_transpose_typed<double>(A, alpha, d_x, beta, d_y, stream)
                                 : spmv_transpose_typed<float>(A, alpha, d_x, beta, d_y, stream);
}

int lapis_paper_vector_length(int64_t nrows, int64_t nnz)
{
    if (nrows <= 0 || nnz < 0) return 1;
    const int64_t mean = (nnz + nrows - 1) / nrows;   // (k + N - 1) / N
    int g = 1;
    while (g < mean && g < LAPIS_WAVE) g *= 2;
    return g;
}

int lapis_spmv_paper_shape(const lapis_csr_t *A, double alpha, const void *d_x, double beta, void *d_y,
                           void *hip_stream)
{
    if (!A) return fail(LAPIS_ERR_INVALID_ARG, "handle is NULL");
    if (A->nrows > 0 && !d_y) return fail(LAPIS_ERR_INVALID_ARG, "d_y is NULL");
    if (A->nnz > 0 && !d_x) return fail(LAPIS_ERR_INVALID_ARG, "d_x is NULL");
    if (A->nrows == 0) return LAPIS_OK;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    return A->dtype == LAPIS_F64 ? spmv_paper_shape_typed<double>(A, alpha, d_x, beta, d_y, stream)
                                 : spmv_paper_shape_typed<float>(A, alpha, d_x, beta, d_y, stream);
}

int lapis_spmm(const lapis_csr_t *A, int64_t k, double alpha, const void *d_X, int64_t ldx, double beta,
               void *d_Y, int64_t ldy, void *hip_stream)
{
    if (!A) return fail(LAPIS_ERR_INVALID_ARG, "handle is NULL");
    if (k <= 0) return fail(LAPIS_ERR_INVALID_ARG, "k must be positive");
    if (ldx < k || ldy < k) return fail(LAPIS_ERR_INVALID_ARG, "leading dimension smaller than k");
    if (A->nrows > 0 && !d_Y) return fail(LAPIS_ERR_INVALID_ARG, "d_Y is NULL");
    if (A->nnz > 0 && !d_X) return fail(LAPIS_ERR_INVALID_ARG, "d_X is NULL");
    if (A->nrows == 0) return LAPIS_OK;
    // one column stored as a plain vector is the matrix-vector product, which has the faster kernels
    if (k == 1 && ldx == 1 && ldy == 1) return lapis_spmv(A, alpha, d_X, beta, d_Y, hip_stream);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    return A->dtype == LAPIS_F64 ? spmm_typed<double>(A, k, alpha, d_X, ldx, beta, d_Y, ldy, stream)
                                 : spmm_typed<float>(A, k, alpha, d_X, ldx, beta, d_Y, ldy, stream);
}

int lapis_csr_destroy(lapis_csr_t *A)
{
    return free_handle(A);
}

int lapis_csr_partition_sizes(const lapis_csr_t *A, int64_t *num_stream, int64_t *num_binned,
                              int64_t *num_long, int64_t *num_tiles)
{
    if (!A) return fail(LAPIS_ERR_INVALID_ARG, "handle is NULL");
    if (num_stream) *num_stream = A->num_stream;
    if (num_binned) *num_binned = A->rows.num_binned;
    if (num_long) *num_long = A->rows.num_long;
    if (num_tiles) *num_tiles = A->rows.num_tiles;
    return LAPIS_OK;
}

int lapis_csr_copy_partition(const lapis_csr_t *A, int32_t *h_stream_chunks, int32_t *h_stream_offset,
                             int32_t *h_bin_offset, int32_t *h_row_perm, int32_t *h_long_off,
                             int32_t *h_tile_row, int32_t *h_tile_nz)
{
    if (!A) return fail(LAPIS_ERR_INVALID_ARG, "handle is NULL");
    LAPIS_HIP(hipDeviceSynchronize());
    if (h_stream_offset) std::memcpy(h_stream_offset, A->h_stream_offset, sizeof(A->h_stream_offset));
    if (h_stream_chunks && A->num_stream > 0)
        LAPIS_HIP(hipMemcpy(h_stream_chunks, A->d_stream_chunks, sizeof(int32_t) * (size_t)A->num_stream, hipMemcpyDeviceToHost));
    return copy_set(A->rows, h_bin_offset, h_row_perm, h_long_off, h_tile_row, h_tile_nz);
}

int lapis_csr_split_sizes(const lapis_csr_t *A, int64_t *num_blocks, int64_t *block_width,
                          int64_t *num_split_rows, int64_t *num_binned, int64_t *num_long,
                          int64_t *num_tiles)
{
    if (!A) return fail(LAPIS_ERR_INVALID_ARG, "handle is NULL");
    if (num_blocks) *num_blocks = A->num_blocks;
    if (block_width) *block_width = A->block_width;
    if (num_split_rows) *num_split_rows = A->num_split;
    if (num_binned) *num_binned = A->vrows.num_binned;
    if (num_long) *num_long = A->vrows.num_long;
    if (num_tiles) *num_tiles = A->vrows.num_tiles;
    return LAPIS_OK;
}

int lapis_csr_copy_split(const lapis_csr_t *A, int32_t *h_cut, int32_t *h_bin_offset, int32_t *h_row_perm,
                         int32_t *h_long_off, int32_t *h_tile_row, int32_t *h_tile_nz)
{
    if (!A) return fail(LAPIS_ERR_INVALID_ARG, "handle is NULL");
    if (A->num_blocks == 0) return fail(LAPIS_ERR_INVALID_ARG, "this matrix has no column split");
    LAPIS_HIP(hipDeviceSynchronize());
    if (h_cut && A->num_split > 0)
        LAPIS_HIP(hipMemcpy(h_cut, A->d_cut, sizeof(int32_t) * (size_t)((A->num_blocks + 1) * A->num_split), hipMemcpyDeviceToHost));
    return copy_set(A->vrows, h_bin_offset, h_row_perm, h_long_off, h_tile_row, h_tile_nz);
}

int lapis_csr_huge_sizes(const lapis_csr_t *A, int64_t *num_huge, int64_t *num_fblocks, int64_t *fblock_width)
{
    if (!A) return fail(LAPIS_ERR_INVALID_ARG, "handle is NULL");
    if (num_huge) *num_huge = A->num_huge;
    if (num_fblocks) *num_fblocks = A->num_fblocks;
    if (fblock_width) *fblock_width = A->fblock_width;
    return LAPIS_OK;
}

int lapis_csr_copy_huge(const lapis_csr_t *A, int32_t *h_split_rows, int32_t *h_huge_rows, int32_t *h_fcut)
{
    if (!A) return fail(LAPIS_ERR_INVALID_ARG, "handle is NULL");
    if (A->num_blocks == 0) return fail(LAPIS_ERR_INVALID_ARG, "this matrix has no column split");
    LAPIS_HIP(hipDeviceSynchronize());
    if (h_split_rows && A->num_split > 0)
        LAPIS_HIP(hipMemcpy(h_split_rows, A->d_split_rows, sizeof(int32_t) * (size_t)A->num_split, hipMemcpyDeviceToHost));
    if (h_huge_rows && A->num_huge > 0)
        LAPIS_HIP(hipMemcpy(h_huge_rows, A->d_huge_rows, sizeof(int32_t) * (size_t)A->num_huge, hipMemcpyDeviceToHost));
    if (h_fcut && A->num_huge > 0)
        LAPIS_HIP(hipMemcpy(h_fcut, A->d_fcut, sizeof(int32_t) * (size_t)((A->num_fblocks + 1) * A->num_huge), hipMemcpyDeviceToHost));
    return LAPIS_OK;
}

int lapis_csr_copy_index16(const lapis_csr_t *A, int *enabled, int64_t *narrow_entries, int64_t *framed_entries,
                           int32_t *h_chunk_base, int32_t *h_frame_table, uint16_t *h_col16)
{
    if (!A) return fail(LAPIS_ERR_INVALID_ARG, "handle is NULL");
    const bool on = A->d_col16 != nullptr;
    if (enabled) *enabled = on ? 1 : 0;
    if (narrow_entries) *narrow_entries = A->narrow_entries;
    if (framed_entries) *framed_entries = A->framed_entries;
    if (!on) return LAPIS_OK;
    LAPIS_HIP(hipDeviceSynchronize());
    if (h_chunk_base && A->num_chunks > 0)
        LAPIS_HIP(hipMemcpy(h_chunk_base, A->d_chunk_base, sizeof(int32_t) * (size_t)A->num_chunks, hipMemcpyDeviceToHost));
    if (h_frame_table && A->num_chunks > 0)
        LAPIS_HIP(hipMemcpy(h_frame_table, A->d_frame_table, sizeof(int32_t) * (size_t)A->num_chunks * kFrameSlots, hipMemcpyDeviceToHost));
    if (h_col16 && A->nnz > 0)
        LAPIS_HIP(hipMemcpy(h_col16, A->d_col16, sizeof(uint16_t) * (size_t)A->nnz, hipMemcpyDeviceToHost));
    return LAPIS_OK;
}

int lapis_csr_copy_patterns(const lapis_csr_t *A, int *enabled, int64_t *pattern_entries, int64_t *pool_size,
                            int32_t *h_pat_off, uint16_t *h_row_pat, int32_t *h_pool)
{
    if (!A) return fail(LAPIS_ERR_INVALID_ARG, "handle is NULL");
    const bool on = A->d_pat_off != nullptr;
    if (enabled) *enabled = on ? 1 : 0;
    if (pattern_entries) *pattern_entries = A->pattern_entries;
    if (pool_size) *pool_size = A->pattern_pool;
    if (!on) return LAPIS_OK;
    LAPIS_HIP(hipDeviceSynchronize());
    if (h_pat_off)
        LAPIS_HIP(hipMemcpy(h_pat_off, A->d_pat_off, sizeof(int32_t) * ((size_t)A->num_chunks + 1), hipMemcpyDeviceToHost));
    if (h_row_pat && A->nrows > 0)
        LAPIS_HIP(hipMemcpy(h_row_pat, A->d_row_pat, sizeof(uint16_t) * (size_t)A->nrows, hipMemcpyDeviceToHost));
    if (h_pool && A->pattern_pool > 0)
        LAPIS_HIP(hipMemcpy(h_pool, A->d_pat_pool, sizeof(int32_t) * (size_t)A->pattern_pool, hipMemcpyDeviceToHost));
    return LAPIS_OK;
}

int lapis_csr_copy_share_classes(const lapis_csr_t *A, int *enabled, int32_t *h_class)
{
    if (!A) return fail(LAPIS_ERR_INVALID_ARG, "handle is NULL");
    const bool on = A->d_share_flag != nullptr;
    if (enabled) *enabled = on ? 1 : 0;
    if (!on || !h_class || A->num_chunks == 0) return LAPIS_OK;
    LAPIS_HIP(hipDeviceSynchronize());
    LAPIS_HIP(hipMemcpy(h_class, A->d_share_flag, sizeof(int32_t) * (size_t)A->num_chunks, hipMemcpyDeviceToHost));
    return LAPIS_OK;
}

int lapis_csr_half_bandwidth(const lapis_csr_t *A, int64_t *half_bandwidth)
{
    if (!A || !half_bandwidth) return fail(LAPIS_ERR_INVALID_ARG, "NULL argument");
    *half_bandwidth = A->half_bandwidth;
    return LAPIS_OK;
}

int lapis_partition_constants(int64_t h_out[10])
{
    if (!h_out) return fail(LAPIS_ERR_INVALID_ARG, "h_out is NULL");
    h_out[0] = LAPIS_NUM_BINS;
    h_out[1] = LAPIS_WAVE;
    h_out[2] = LAPIS_LONG_THRESHOLD;
    h_out[3] = LAPIS_TILE_NNZ;
    h_out[4] = LAPIS_STREAM_ROWS;
    h_out[5] = LAPIS_STREAM_MIN_NNZ;
    h_out[6] = LAPIS_SPLIT_BLOCK_BYTES;
    h_out[7] = LAPIS_SPLIT_MAX_BLOCKS;
    h_out[8] = LAPIS_HUGE_ROW;
    h_out[9] = LAPIS_LDS_BLOCK_BYTES;
    return LAPIS_OK;
}

const char *lapis_last_error(void)
{
    return g_last_error.c_str();
}

}  // extern "C"
