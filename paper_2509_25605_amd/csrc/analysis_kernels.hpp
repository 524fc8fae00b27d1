// Row-partition analysis on the device.  First, chunks of consecutive rows that
// are short throughout and hold enough entries are marked as stream chunks.
// The other rows get the per-row form of the vector-length estimate of
// Section 4.2 ("Parallelism estimation": entries per row, rounded up, clamped
// to the hardware vector width): each row gets the bin of its own length, rows
// are listed per bin in ascending order, and the rows beyond the long threshold
// are cut into equal tiles of entries.  All results
// are integers with a unique value, produced without atomics on ordered data,
// so they can be compared bit for bit with a CPU reference.
#pragma once
#include "device_utils.hpp"

namespace lapis {

constexpr int kNumBins = 10;
constexpr int kRowsPerThread = 8;
constexpr int kRowsPerAnalysisBlock = kBlock * kRowsPerThread;  // 2048 rows per workgroup

template <int LONG_THRESHOLD>
__device__ __forceinline__ int bin_of_length(int32_t len)
{
    if (len <= 0) return 0;
    if (len == 1) return 1;
    if (len <= kWave) return 33 - __clz(len - 1);  // 1 + ceil(log2(len))
    return len <= LONG_THRESHOLD ? 8 : 9;
}

// Exclusive scan of one int per thread across the workgroup; returns the
// thread's prefix and writes the workgroup total to *total.
__device__ __forceinline__ int32_t block_exclusive_scan(int32_t v, int32_t *s_tmp, int32_t *total)
{
    // s_tmp: kBlock ints.  Hillis-Steele inclusive scan in LDS.
    s_tmp[threadIdx.x] = v;
    __syncthreads();
    for (int d = 1; d < kBlock; d <<= 1) {
        int32_t add = (threadIdx.x >= (unsigned)d) ? s_tmp[threadIdx.x - d] : 0;
        __syncthreads();
        s_tmp[threadIdx.x] += add;
        __syncthreads();
    }
    const int32_t incl = s_tmp[threadIdx.x];
    *total = s_tmp[kBlock - 1];
    __syncthreads();
    return incl - v;
}

// Pass 0a: flag[c] = class of chunk c (chunk_rows consecutive rows): 0 if the chunk holds fewer
// than min_nnz entries or a row has more than 16*chunk_rows entries, else the smallest k in 1..4
// with (longest row) <= 2^k * chunk_rows and (entries) <= 2^k * 16 * chunk_rows (the length
// condition alone if no k meets the second one).
__global__ __launch_bounds__(kBlock) void chunk_flag_kernel(int32_t nrows, int32_t num_chunks,
                                                            int32_t chunk_rows, int32_t min_nnz,
                                                            const int32_t *__restrict__ rowptr,
                                                            int32_t *__restrict__ flag)
{
    const int64_t c = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (c >= num_chunks) return;
    const int64_t first = c * chunk_rows;
    const int64_t last = (first + chunk_rows < nrows) ? first + chunk_rows : nrows;
    int32_t prev = rowptr[first];
    const int32_t begin = prev;
    int32_t longest = 0;
    for (int64_t i = first + 1; i <= last; ++i) {
        const int32_t cur = rowptr[i];
        longest = (cur - prev > longest) ? cur - prev : longest;
        prev = cur;
    }
    int cls = 0;
    const int32_t entries = prev - begin;
    if (entries >= min_nnz) {
        for (int k = 4; k >= 1; --k)
            if (longest <= (chunk_rows << k)) cls = k;
        if (cls) {
            int fit = 0;
            for (int k = 4; k >= cls; --k)
                if (entries <= ((chunk_rows * 16) << k)) fit = k;
            if (fit) cls = fit;
        }
    }
    flag[c] = cls;
}

// Pass 0b, three launches (histogram per block of kCompactBlock chunks, scan, ordered scatter):
// list = the chunk ids of class 1, then of class 2, ... each class ascending; offset[k] =
// position of the first chunk of class k+1, offset[kChunkClasses] = number of listed chunks.
// flag holds values 0..kChunkClasses.
constexpr int kChunkClasses = 4;
constexpr int kCompactBlock = 1024;
// Step 1 of 3: hist[b * kChunkClasses + k - 1] = how many of the chunks b * kCompactBlock ..
// (b + 1) * kCompactBlock - 1 are of class k.
__global__ __launch_bounds__(kCompactBlock) void chunk_class_hist_kernel(int32_t num_chunks,
                                                                         const int32_t *__restrict__ flag,
                                                                         int32_t *__restrict__ hist)
{
    __shared__ int32_t s_count[kChunkClasses];
    if (threadIdx.x < kChunkClasses) s_count[threadIdx.x] = 0;
    __syncthreads();
    const int64_t c = (int64_t)blockIdx.x * kCompactBlock + threadIdx.x;
    const int32_t f = (c < num_chunks) ? flag[c] : 0;
#pragma unroll
    for (int k = 0; k < kChunkClasses; ++k) {
        const uint64_t m = __builtin_amdgcn_ballot_w64(f == k + 1);
        if (threadIdx.x % kWave == 0 && m) atomicAdd(&s_count[k], (int32_t)__popcll(m));
    }
    __syncthreads();
    if (threadIdx.x < kChunkClasses) hist[(int64_t)blockIdx.x * kChunkClasses + threadIdx.x] = s_count[threadIdx.x];
}

// Step 2 of 3, one workgroup: offset[0 .. kChunkClasses] = where each class's list starts in
// `list` (and the total), and hist[b * kChunkClasses + k - 1] becomes where the class-k chunks of
// block b go: the class's start plus the class-k chunks of the blocks before b.
__global__ __launch_bounds__(kCompactBlock) void chunk_class_scan_kernel(int32_t num_blocks, int32_t *__restrict__ hist,
                                                                         int32_t *__restrict__ offset)
{
    __shared__ int32_t s_part[kCompactBlock];
    __shared__ int32_t s_total[kChunkClasses + 1];
    const int tid = threadIdx.x;
    const int32_t per = (num_blocks + kCompactBlock - 1) / kCompactBlock;
    const int32_t b0 = tid * per, b1 = (b0 + per < num_blocks) ? b0 + per : num_blocks;
    if (tid == 0) s_total[0] = 0;
    for (int k = 0; k < kChunkClasses; ++k) {
        int32_t sum = 0;
        for (int32_t b = b0; b < b1; ++b) sum += hist[(int64_t)b * kChunkClasses + k];
        __syncthreads();
        s_part[tid] = sum;
        __syncthreads();
        for (int d = 1; d < kCompactBlock; d *= 2) {
            const int32_t other = tid >= d ? s_part[tid - d] : 0;
            __syncthreads();
            s_part[tid] += other;
            __syncthreads();
        }
        if (tid == kCompactBlock - 1) s_total[k + 1] = s_total[k] + s_part[tid];
        __syncthreads();
        int32_t at = s_total[k] + s_part[tid] - sum;       // exclusive prefix of this thread's blocks
        for (int32_t b = b0; b < b1; ++b) {
            const int32_t n = hist[(int64_t)b * kChunkClasses + k];
            hist[(int64_t)b * kChunkClasses + k] = at;
            at += n;
        }
    }
    __syncthreads();
    if (tid <= kChunkClasses) offset[tid] = s_total[tid];
}

// Step 3 of 3: list[] = the chunks of class 1, then class 2, ..., each ascending; start[] is
// the hist[] that step 2 left.  Ballots give the position inside the wavefront, LDS the counts
// of the wavefronts before it.
__global__ __launch_bounds__(kCompactBlock) void chunk_compact_kernel(int32_t num_chunks,
                                                                      const int32_t *__restrict__ flag,
                                                                      const int32_t *__restrict__ start,
                                                                      int32_t *__restrict__ list)
{
    constexpr int kWaves = kCompactBlock / kWave;
    __shared__ int32_t s_wave[kWaves][kChunkClasses];
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int64_t c = (int64_t)blockIdx.x * kCompactBlock + threadIdx.x;
    const int32_t f = (c < num_chunks) ? flag[c] : 0;
    uint64_t mine = 0;
#pragma unroll
    for (int k = 0; k < kChunkClasses; ++k) {
        const uint64_t m = __builtin_amdgcn_ballot_w64(f == k + 1);
        if (lane == 0) s_wave[wave][k] = __popcll(m);
        if (f == k + 1) mine = m;
    }
    __syncthreads();
    if (f) {
        int32_t before = start[(int64_t)blockIdx.x * kChunkClasses + f - 1];
        for (int w = 0; w < wave; ++w) before += s_wave[w][f - 1];
        list[before + __popcll(mine & ((1ull << lane) - 1))] = (int32_t)c;
    }
}

// flag[c] = 0 for every stream chunk that is neither narrow nor framed (chunk_base == -1) and has a
// row of more than `wave` entries: its rows go to the bins instead.
__global__ __launch_bounds__(kBlock) void chunk_demote_kernel(int32_t nrows, int32_t num_chunks, int32_t chunk_rows,
                                                              int32_t wave, const int32_t *__restrict__ rowptr,
                                                              const int32_t *__restrict__ chunk_base,
                                                              int32_t *__restrict__ flag)
{
    const int64_t c = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (c >= num_chunks || flag[c] == 0 || chunk_base[c] != -1) return;
    const int64_t first = c * chunk_rows;
    const int64_t last = (first + chunk_rows < nrows) ? first + chunk_rows : nrows;
    int32_t prev = rowptr[first], longest = 0;
    for (int64_t i = first + 1; i <= last; ++i) {
        const int32_t cur = rowptr[i];
        longest = (cur - prev > longest) ? cur - prev : longest;
        prev = cur;
    }
    if (longest > wave) flag[c] = 0;
}

// Level 1b, one wavefront per chunk: chunk_base[c] = smallest column of stream chunk c if its
// columns span at most 65535, else -1 (also for chunks that are not stream chunks);
// The totals are taken by narrow_count_kernel (one atomic per chunk on one address would
// serialise: it cost 1 ms on 65 536 chunks).
__global__ __launch_bounds__(kBlock) void chunk_span_kernel(int32_t nrows, int32_t num_chunks, int32_t chunk_rows,
                                                            const int32_t *__restrict__ chunk_flag,
                                                            const int32_t *__restrict__ rowptr,
                                                            const int32_t *__restrict__ colidx,
                                                            int32_t *__restrict__ chunk_base)
{
    const int64_t c = (int64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
    const int lane = threadIdx.x % kWave;
    if (c >= num_chunks) return;                       // whole wavefronts leave together
    if (chunk_flag[c] == 0) {
        if (lane == 0) chunk_base[c] = -1;
        return;
    }
    const int64_t first = c * chunk_rows;
    const int64_t last = (first + chunk_rows < nrows) ? first + chunk_rows : nrows;
    const int32_t b = rowptr[first], e = rowptr[last];
    int32_t hi = 0, lo_rev = 0;                        // lo_rev = INT32_MAX - smallest column
    for (int32_t j = b + lane; j < e; j += 8 * kWave) {     // 8 loads in flight; past the end: the last entry again
        int32_t col[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) col[q] = load_stream(colidx + (j + q * kWave < e ? j + q * kWave : e - 1));
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            hi = max(hi, col[q]);
            lo_rev = max(lo_rev, INT32_MAX - col[q]);
        }
    }
    hi = wave_max_nonneg(hi);
    const int32_t lo = INT32_MAX - wave_max_nonneg(lo_rev);
    if (lane == 0) {
        const bool narrow = e > b && hi - lo <= 65535;
        chunk_base[c] = narrow ? lo : -1;
    }
}

// Totals over the chunks, added to entries_out / narrow_chunks (zero on entry; any number of
// workgroups of kCompactBlock threads): entries[0] = entries of the narrow chunks (chunk_base >= 0),
// entries[1] = entries of the framed chunks (chunk_base == -2), entries[2] = entries of the
// patterned stream chunks (pat_len > 0), entries[3] = sum of their table lengths,
// entries[4 + k - 1] / entries[4 + kChunkClasses + k - 1] = the last two for class k alone;
// narrow_chunks[q * kChunkClasses + k - 1] = how many chunks of class k are narrow (q = 0), framed
// (1), patterned (2), patterned or narrow or framed (3).
__global__ __launch_bounds__(kCompactBlock) void narrow_count_kernel(int32_t nrows, int32_t num_chunks,
                                                                     int32_t chunk_rows,
                                                                     const int32_t *__restrict__ chunk_flag,
                                                                     const int32_t *__restrict__ rowptr,
                                                                     const int32_t *__restrict__ chunk_base,
                                                                     const int32_t *__restrict__ pat_len,
                                                                     unsigned long long *__restrict__ entries_out,
                                                                     int32_t *__restrict__ narrow_chunks)
{
    constexpr int kTotals = 4 + 2 * kChunkClasses;
    __shared__ unsigned long long s_entries[kTotals];
    __shared__ int32_t s_chunks[4 * kChunkClasses];
    if (threadIdx.x < kTotals) s_entries[threadIdx.x] = 0;
    if (threadIdx.x < 4 * kChunkClasses) s_chunks[threadIdx.x] = 0;
    __syncthreads();
    unsigned long long entries = 0, framed = 0, patterned = 0, table = 0;
    unsigned long long cls_entries[kChunkClasses] = {0, 0, 0, 0}, cls_table[kChunkClasses] = {0, 0, 0, 0};
    int32_t chunks[4 * kChunkClasses] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    for (int64_t c = (int64_t)blockIdx.x * kCompactBlock + threadIdx.x; c < num_chunks; c += (int64_t)gridDim.x * kCompactBlock) {
        const int32_t base = chunk_base[c];
        const int32_t cls = chunk_flag[c];
        const int32_t plen = cls != 0 ? pat_len[c] : 0;
        if (base == -1 && plen == 0) continue;
        const int64_t first = c * chunk_rows;
        const int64_t last = (first + chunk_rows < nrows) ? first + chunk_rows : nrows;
        const unsigned long long len = (unsigned long long)(rowptr[last] - rowptr[first]);
        if (base == -2) framed += len; else if (base >= 0) entries += len;
        if (plen > 0) { patterned += len; table += (unsigned long long)plen; }
#pragma unroll
        for (int k = 0; k < kChunkClasses; ++k) {
            if (cls == k + 1 && plen > 0) { cls_entries[k] += len; cls_table[k] += (unsigned long long)plen; }
            chunks[k] += (cls == k + 1 && base >= 0);
            chunks[kChunkClasses + k] += (cls == k + 1 && base == -2);
            chunks[2 * kChunkClasses + k] += (cls == k + 1 && plen > 0);
            chunks[3 * kChunkClasses + k] += (cls == k + 1 && (plen > 0 || base != -1));
        }
    }
    if (entries) atomicAdd(&s_entries[0], entries);
    if (framed) atomicAdd(&s_entries[1], framed);
    if (patterned) atomicAdd(&s_entries[2], patterned);
    if (table) atomicAdd(&s_entries[3], table);
#pragma unroll
    for (int k = 0; k < kChunkClasses; ++k) {
        if (cls_entries[k]) atomicAdd(&s_entries[4 + k], cls_entries[k]);
        if (cls_table[k]) atomicAdd(&s_entries[4 + kChunkClasses + k], cls_table[k]);
    }
#pragma unroll
    for (int k = 0; k < 4 * kChunkClasses; ++k)
        if (chunks[k]) atomicAdd(&s_chunks[k], chunks[k]);
    __syncthreads();
    if (threadIdx.x < kTotals && s_entries[threadIdx.x]) atomicAdd(&entries_out[threadIdx.x], s_entries[threadIdx.x]);
    if (threadIdx.x < 4 * kChunkClasses && s_chunks[threadIdx.x]) atomicAdd(&narrow_chunks[threadIdx.x], s_chunks[threadIdx.x]);
}

// Frames of 2048 columns for the stream chunks that are not narrow (chunk_base == -1 on entry),
// one wavefront per chunk: the distinct frames (column >> 11) are taken out smallest first; with
// at most 32 of them the chunk becomes "framed": chunk_base = -2 and frame_table[32*c + k] = the
// k-th smallest frame (the largest one repeated above the count).  frame_table must be 0 on entry.
// Where the chunk's frames span fewer than kFrameBitmapBits they are marked in a bitmap (two
// passes over the entries in all); otherwise every frame taken out costs a pass.
constexpr int kAnalysisFrameShift = 11;
constexpr int kAnalysisFrameSlots = 32;
constexpr int kFrameBitmapBits = 8192;     // widest range of frames (16.8 M columns) handled with a bitmap in LDS
__global__ __launch_bounds__(kBlock) void chunk_frames_kernel(int32_t nrows, int32_t num_chunks, int32_t chunk_rows,
                                                              const int32_t *__restrict__ chunk_flag,
                                                              const int32_t *__restrict__ rowptr,
                                                              const int32_t *__restrict__ colidx,
                                                              int32_t *__restrict__ chunk_base,
                                                              int32_t *__restrict__ frame_table)
{
    const int64_t c = (int64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
    const int lane = threadIdx.x % kWave;
    if (c >= num_chunks) return;                       // whole wavefronts leave together
    if (chunk_flag[c] == 0 || chunk_base[c] != -1) return;
    const int64_t first = c * chunk_rows;
    const int64_t last_row = (first + chunk_rows < nrows) ? first + chunk_rows : nrows;
    const int32_t b = rowptr[first], e = rowptr[last_row];
    // smallest and largest frame of the chunk
    int32_t rev_lo = 0, hi = 0;
    for (int32_t j = b + lane; j < e; j += kWave) {
        const int32_t f = load_stream(colidx + j) >> kAnalysisFrameShift;
        rev_lo = max(rev_lo, INT32_MAX - f);
        hi = max(hi, f);
    }
    rev_lo = wave_max_nonneg(rev_lo);
    hi = wave_max_nonneg(hi);
    if (rev_lo == 0) return;                           // no entries (cannot happen for a flagged chunk)
    const int32_t lo = INT32_MAX - rev_lo;
    int32_t last = -1, mine = 0, count = 0;
    if (hi - lo < kFrameBitmapBits) {
        // one more pass marks the frames in a bitmap in LDS; the set bits in ascending order are the table
        __shared__ uint32_t s_bits[kWavesPerBlock][kFrameBitmapBits / 32];
        uint32_t *bits = s_bits[threadIdx.x / kWave];
        constexpr int kWordsPerLane = kFrameBitmapBits / 32 / kWave;
#pragma unroll
        for (int q = 0; q < kWordsPerLane; ++q) bits[lane * kWordsPerLane + q] = 0;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        for (int32_t j = b + lane; j < e; j += kWave) {
            const int32_t f = (load_stream(colidx + j) >> kAnalysisFrameShift) - lo;
            atomicOr(&bits[f >> 5], 1u << (f & 31));
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        uint32_t word[kWordsPerLane];
        int32_t set = 0;
#pragma unroll
        for (int q = 0; q < kWordsPerLane; ++q) {
            word[q] = bits[lane * kWordsPerLane + q];
            set += __popc(word[q]);
        }
        count = 0;
        for (int d = 0; d < kWave; ++d) count += __builtin_amdgcn_readlane(set, d);
        if (count > kAnalysisFrameSlots) return;       // too scattered: stays -1
        for (int k = 0; k < count; ++k) {              // uniform: the k-th smallest marked frame
            int32_t rev = 0;
#pragma unroll
            for (int q = kWordsPerLane - 1; q >= 0; --q) {
                if (word[q]) rev = INT32_MAX - (lo + (lane * kWordsPerLane + q) * 32 + (__ffs(word[q]) - 1));
            }
            rev = wave_max_nonneg(rev);
            last = INT32_MAX - rev;
            if (lane == k) mine = last;
            const int32_t at = last - lo;              // clear it in the lane that holds it
#pragma unroll
            for (int q = 0; q < kWordsPerLane; ++q)
                if ((at >> 5) == lane * kWordsPerLane + q) word[q] &= ~(1u << (at & 31));
        }
    } else {
        for (int k = 0; k <= kAnalysisFrameSlots; ++k) {
            int32_t rev = 0;                           // INT32_MAX - (smallest frame above `last` seen by this lane)
            for (int32_t j = b + lane; j < e; j += kWave) {
                const int32_t f = colidx[j] >> kAnalysisFrameShift;
                if (f > last) rev = max(rev, INT32_MAX - f);
            }
            rev = wave_max_nonneg(rev);
            if (rev == 0) break;                       // no frame left
            if (k == kAnalysisFrameSlots) { count = kAnalysisFrameSlots + 1; break; }
            last = INT32_MAX - rev;
            if (lane == k) mine = last;
            count = k + 1;
        }
        if (count > kAnalysisFrameSlots) return;       // too scattered: stays -1
    }
    if (lane < kAnalysisFrameSlots) frame_table[c * kAnalysisFrameSlots + lane] = lane < count ? mine : last;
    if (lane == 0) chunk_base[c] = -2;
}

// col16[j] for the entries of the narrow chunks (colidx[j] - chunk_base[c]) and of the framed
// chunks ((rank of the entry's frame in the chunk's table) << 11 | (colidx[j] & 2047)); col16 is
// 0 elsewhere.  One wavefront per chunk.
__global__ __launch_bounds__(kBlock) void col16_fill_kernel(int32_t nrows, int32_t num_chunks, int32_t chunk_rows,
                                                            const int32_t *__restrict__ rowptr,
                                                            const int32_t *__restrict__ colidx,
                                                            const int32_t *__restrict__ chunk_base,
                                                            const int32_t *__restrict__ frame_table,
                                                            uint16_t *__restrict__ col16)
{
    const int64_t c = (int64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
    const int lane = threadIdx.x % kWave;
    if (c >= num_chunks) return;
    const int32_t base = chunk_base[c];
    if (base == -1) return;
    const int64_t first = c * chunk_rows;
    const int64_t last = (first + chunk_rows < nrows) ? first + chunk_rows : nrows;
    const int32_t e = rowptr[last];
    if (base >= 0) {
        for (int32_t j = rowptr[first] + lane; j < e; j += kWave) col16[j] = (uint16_t)(load_stream(colidx + j) - base);
        return;
    }
    // framed: lane t < 32 keeps table entry t; the rank of a frame is the number of entries below it
    const int32_t tab = frame_table[c * kAnalysisFrameSlots + (lane % kAnalysisFrameSlots)];
    for (int32_t j0 = rowptr[first]; j0 < e; j0 += kWave) {           // uniform trip count: readlane needs all lanes
        const int32_t j = j0 + lane;
        const int32_t col = j < e ? load_stream(colidx + j) : 0;
        const int32_t f = col >> kAnalysisFrameShift;
        int32_t rank = 0;
#pragma unroll
        for (int t = 0; t < kAnalysisFrameSlots; ++t) rank += (__builtin_amdgcn_readlane(tab, t) < f);
        if (j < e) col16[j] = (uint16_t)((rank << kAnalysisFrameShift) | (col & ((1 << kAnalysisFrameShift) - 1)));
    }
}

// Level 1c, one wavefront per chunk: the row patterns of a stream chunk.  The list of a
// non-empty row i is its diagonals colidx[j] - i in stored order, its shape that list minus its
// first element.  Going through the rows in ascending order, a row takes the first stored list
// (in order of insertion) with its length, its shape and a shift = (its first diagonal) - (the
// stored list's first diagonal) in [-64, 63]; a row that finds none appends its own list to the
// chunk's table (LDS here), shift 0.  row_pat[i] = (where the taken list starts in the table) |
// ((shift & 127) << 9), 0 for empty rows.
// pat_len[c] = length of the table if no row has more than kPatternMaxRow entries, at most
// kPatternSlots patterns were needed, the table has at most kPatternTableSize diagonals and
// twice its length does not exceed the chunk's entries; otherwise 0 (and row_pat 0 for the
// chunk's rows).  Chunks that do not stream get 0 as well.  chunk_rows divides 64.
constexpr int kPatternMaxRow = 128, kPatternSlots = 8, kPatternTableSize = 512;
constexpr int kPatternShiftBit = 9, kPatternShiftMax = 63;     // row_pat: start in bits 0..8, shift (-64..63) in bits 9..15
static_assert(kPatternTableSize == 1 << kPatternShiftBit, "a start fits below the shift bits");
__global__ __launch_bounds__(kBlock) void chunk_patterns_kernel(int32_t nrows, int32_t num_chunks, int32_t chunk_rows,
                                                                const int32_t *__restrict__ chunk_flag,
                                                                const int32_t *__restrict__ rowptr,
                                                                const int32_t *__restrict__ colidx,
                                                                int32_t *__restrict__ pat_len,
                                                                uint16_t *__restrict__ row_pat)
{
    static_assert(kPatternMaxRow == 2 * kWave, "two entries of a row per lane");
    __shared__ int32_t s_table[kWavesPerBlock][kPatternTableSize];
    const int64_t c = (int64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
    const int lane = threadIdx.x % kWave;
    if (c >= num_chunks) return;                       // whole wavefronts leave together
    const int64_t first = c * chunk_rows;
    const int64_t last = (first + chunk_rows < nrows) ? first + chunk_rows : nrows;
    int32_t *tab = s_table[threadIdx.x / kWave];
    int32_t p_start[kPatternSlots], p_len[kPatternSlots];
#pragma unroll
    for (int p = 0; p < kPatternSlots; ++p) { p_start[p] = 0; p_len[p] = 0; }
    int32_t P = 0, L = 0, mine = 0;
    bool ok = chunk_flag[c] != 0;
    // Most rows repeat the row before them (its columns shifted by one).  That is settled first
    // for all rows at once, kWave / chunk_rows lanes per row striding its entries; only the rows
    // that differ from their predecessor go through the comparison with the stored lists below,
    // the others take their predecessor's answer (the same list, so the same place in the table).
    const int per_row = kWave / chunk_rows;
    const int64_t r_mine = first + lane / per_row;
    const bool has_row = ok && lane / per_row < chunk_rows && r_mine < last;
    const int32_t b_mine = has_row ? rowptr[r_mine] : 0;
    const int32_t len_mine = has_row ? rowptr[r_mine + 1] - b_mine : 0;
    const int32_t b_prev = (has_row && r_mine > first) ? rowptr[r_mine - 1] : b_mine;
    bool repeats = has_row && r_mine > first && len_mine > 0 && b_mine - b_prev == len_mine;
    const int32_t longest = wave_max_nonneg(len_mine);
    if (longest > kPatternMaxRow) ok = false;
    if (ok) {
        for (int32_t k = lane % per_row; k < longest; k += per_row)
            if (repeats && k < len_mine) repeats = colidx[b_mine + k] - colidx[b_prev + k] == 1;
    }
    // bit r of `search`: row first + r has entries and does not repeat its predecessor
    unsigned long long search = 0;
    {
        const unsigned long long differs = __ballot(has_row && len_mine > 0 && !repeats);   // per lane
        for (int r = 0; r < chunk_rows; ++r)
            if ((differs >> (r * per_row)) & ((1ull << per_row) - 1)) search |= 1ull << r;
    }
    const unsigned long long nonempty_lanes = __ballot(has_row && len_mine > 0);
    for (unsigned long long todo = ok ? search : 0; todo != 0 && ok; todo &= todo - 1) {     // uniform
        const int t = __builtin_ctzll(todo);
        const int64_t r = first + t;
        const int32_t b = __builtin_amdgcn_readlane(b_mine, t * per_row);
        const int32_t len = __builtin_amdgcn_readlane(len_mine, t * per_row);
        const int32_t d0 = lane < len ? colidx[b + lane] - (int32_t)r : 0;
        const int32_t d1 = lane + kWave < len ? colidx[b + kWave + lane] - (int32_t)r : 0;
        const int32_t head = __builtin_amdgcn_readfirstlane(d0);          // the row's first diagonal (len >= 1)
        int32_t found = -1, found_shift = 0;
#pragma unroll
        for (int p = 0; p < kPatternSlots; ++p) {
            if (found < 0 && p < P && p_len[p] == len) {
                const int32_t shift = head - tab[p_start[p]];              // uniform
                if (shift >= -kPatternShiftMax - 1 && shift <= kPatternShiftMax) {
                    const bool same = (lane >= len || tab[p_start[p] + lane] + shift == d0) &&
                                      (lane + kWave >= len || tab[p_start[p] + kWave + lane] + shift == d1);
                    if (__ballot(!same) == 0) { found = p_start[p]; found_shift = shift; }
                }
            }
        }
        if (found < 0) {
            if (P == kPatternSlots || L + len > kPatternTableSize) { ok = false; break; }
            if (lane < len) tab[L + lane] = d0;
            if (lane + kWave < len) tab[L + kWave + lane] = d1;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int p = 0; p < kPatternSlots; ++p)
                if (p == P) { p_start[p] = L; p_len[p] = len; }
            found = L;
            P += 1;
            L += len;
        }
        if (lane == t) mine = found | ((found_shift & (2 * kPatternShiftMax + 1)) << kPatternShiftBit);
    }
    // lane r < chunk_rows answers for row first + r: a row that repeats its predecessor takes the
    // answer of the nearest searched row below it; empty rows keep 0
    {
        const bool my_nonempty = lane < chunk_rows && ((nonempty_lanes >> (lane * per_row)) & 1);
        const unsigned long long below = lane < chunk_rows ? (search & ((2ull << lane) - 1)) : 0;
        const int src = below ? 63 - __builtin_clzll(below) : 0;
        const int32_t taken = __shfl(mine, src, kWave);
        mine = (my_nonempty && below) ? taken : 0;
    }
    const int32_t entries = rowptr[last] - rowptr[first];
    if (!ok || 2 * L > entries) { L = 0; mine = 0; }
    if (lane == 0) pat_len[c] = L;
    if (lane < chunk_rows && first + lane < last) row_pat[first + lane] = (uint16_t)mine;
}

// The tables of the patterned chunks back to back: pool[pat_off[c] + start + k] = diagonal of the
// k-th entry of the first row of the chunk whose row_pat has that start (the row that stored the
// list: its shift is 0).  One wavefront per chunk; chunk_rows <= 64.
__global__ __launch_bounds__(kBlock) void pattern_pool_kernel(int32_t nrows, int32_t num_chunks, int32_t chunk_rows,
                                                              const int32_t *__restrict__ rowptr,
                                                              const int32_t *__restrict__ colidx,
                                                              const int32_t *__restrict__ pat_off,
                                                              const uint16_t *__restrict__ row_pat,
                                                              int32_t *__restrict__ pool)
{
    const int64_t c = (int64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
    const int lane = threadIdx.x % kWave;
    if (c >= num_chunks) return;
    const int32_t off = pat_off[c];
    if (pat_off[c + 1] == off) return;
    // only the first row with each list writes it: lane r looks after row first + r
    const int64_t first = c * (int64_t)chunk_rows;
    const int64_t r = first + lane;
    const bool has_row = lane < chunk_rows && r < nrows;
    const int32_t b = has_row ? rowptr[r] : 0;
    const int32_t len = has_row ? rowptr[r + 1] - b : 0;
    const int32_t start = has_row ? (int32_t)row_pat[r] & (kPatternTableSize - 1) : 0;    // without the shift bits
    bool writer = len > 0;
    for (int t = 0; t < chunk_rows; ++t) {             // uniform
        const int32_t t_start = __builtin_amdgcn_readlane(start, t);
        const int32_t t_len = __builtin_amdgcn_readlane(len, t);
        if (t < lane && t_len > 0 && t_start == start) writer = false;
    }
    unsigned long long todo = __ballot(writer);
    while (todo) {                                     // uniform: at most kPatternSlots rows
        const int t = __builtin_ctzll(todo);
        todo &= todo - 1;
        const int32_t t_b = __builtin_amdgcn_readlane(b, t);
        const int32_t t_len = __builtin_amdgcn_readlane(len, t);
        const int32_t at = off + __builtin_amdgcn_readlane(start, t);
        for (int32_t k = lane; k < t_len; k += kWave) pool[at + k] = colidx[t_b + k] - (int32_t)(first + t);
    }
}

// Pass 1: per-workgroup histogram of row bins (rows of flagged chunks are skipped; chunk_flag
// may be null); hist is bin-major: hist[bin*num_blocks + block].  row_begin[i] / row_end[i]
// delimit row i: (rowptr, rowptr + 1) for the matrix's rows, the cut table for virtual rows.
template <int LONG_THRESHOLD>
__global__ __launch_bounds__(kBlock) void bin_count_kernel(int32_t nrows,
                                                           const int32_t *__restrict__ row_begin,
                                                           const int32_t *__restrict__ row_end,
                                                           int32_t chunk_rows,
                                                           const int32_t *__restrict__ chunk_flag,
                                                           int32_t num_blocks,
                                                           int32_t *__restrict__ hist)
{
    __shared__ int32_t s_hist[kNumBins];
    if (threadIdx.x < kNumBins) s_hist[threadIdx.x] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * kRowsPerAnalysisBlock;
    for (int it = 0; it < kRowsPerThread; ++it) {
        const int64_t i = base + (int64_t)it * kBlock + threadIdx.x;
        if (i < nrows && !(chunk_flag && chunk_flag[i / chunk_rows]))
            atomicAdd(&s_hist[bin_of_length<LONG_THRESHOLD>(row_end[i] - row_begin[i])], 1);
    }
    __syncthreads();
    if (threadIdx.x < kNumBins) hist[(int64_t)threadIdx.x * num_blocks + blockIdx.x] = s_hist[threadIdx.x];
}

// Pass 2 (one workgroup): exclusive scan of hist in place, in bin-major order,
// so hist[bin*num_blocks + block] becomes the first position in row_perm of the
// rows of `bin` found by `block`; also bin_offset[0..kNumBins].
__global__ __launch_bounds__(kBlock) void bin_scan_kernel(int64_t count, int32_t num_blocks,
                                                          int32_t *__restrict__ hist,
                                                          int32_t *__restrict__ bin_offset)
{
    __shared__ int32_t s_tmp[kBlock];
    int32_t running = 0;
    for (int64_t base = 0; base < count; base += kBlock) {
        const int64_t i = base + threadIdx.x;
        const int32_t v = (i < count) ? hist[i] : 0;
        int32_t total;
        const int32_t excl = block_exclusive_scan(v, s_tmp, &total);
        if (i < count) {
            hist[i] = running + excl;
            if (i % num_blocks == 0) bin_offset[i / num_blocks] = running + excl;
        }
        running += total;
    }
    if (threadIdx.x == 0) bin_offset[kNumBins] = running;
}

// Pass 3: stable scatter of row ids into row_perm.
template <int LONG_THRESHOLD>
__global__ __launch_bounds__(kBlock) void bin_scatter_kernel(int32_t nrows,
                                                             const int32_t *__restrict__ row_begin,
                                                             const int32_t *__restrict__ row_end,
                                                             int32_t chunk_rows,
                                                             const int32_t *__restrict__ chunk_flag,
                                                             int32_t num_blocks,
                                                             const int32_t *__restrict__ hist,
                                                             int32_t *__restrict__ row_perm)
{
    __shared__ int32_t s_base[kNumBins];                     // next free position per bin
    __shared__ int32_t s_wave[kWavesPerBlock][kNumBins];     // per-wave counts of this pass
    if (threadIdx.x < kNumBins) s_base[threadIdx.x] = hist[(int64_t)threadIdx.x * num_blocks + blockIdx.x];
    __syncthreads();
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int64_t base = (int64_t)blockIdx.x * kRowsPerAnalysisBlock;
    for (int it = 0; it < kRowsPerThread; ++it) {
        const int64_t i = base + (int64_t)it * kBlock + threadIdx.x;
        const int bin = (i < nrows && !(chunk_flag && chunk_flag[i / chunk_rows]))
                            ? bin_of_length<LONG_THRESHOLD>(row_end[i] - row_begin[i]) : -1;
        int32_t rank_in_wave = 0;
        for (int b = 0; b < kNumBins; ++b) {
            const uint64_t mask = __ballot(bin == b);
            if (bin == b) rank_in_wave = __popcll(mask & ((1ull << lane) - 1));
            if (lane == 0) s_wave[wave][b] = __popcll(mask);
        }
        __syncthreads();
        if (bin >= 0) {
            int32_t pos = s_base[bin] + rank_in_wave;
            for (int w = 0; w < wave; ++w) pos += s_wave[w][bin];
            row_perm[pos] = (int32_t)i;
        }
        __syncthreads();
        if (threadIdx.x < kNumBins) {
            int32_t add = 0;
            for (int w = 0; w < kWavesPerBlock; ++w) add += s_wave[w][threadIdx.x];
            s_base[threadIdx.x] += add;
        }
        __syncthreads();
    }
}

// Pass 4 (one workgroup): long_off[0..m] = exclusive scan of the long rows' lengths.
__global__ __launch_bounds__(kBlock) void long_scan_kernel(int32_t m, const int32_t *__restrict__ long_rows,
                                                           const int32_t *__restrict__ row_begin,
                                                           const int32_t *__restrict__ row_end,
                                                           int32_t *__restrict__ long_off)
{
    __shared__ int32_t s_tmp[kBlock];
    int32_t running = 0;
    for (int64_t base = 0; base < m; base += kBlock) {
        const int64_t r = base + threadIdx.x;
        int32_t v = 0;
        if (r < m) { const int32_t row = long_rows[r]; v = row_end[row] - row_begin[row]; }
        int32_t total;
        const int32_t excl = block_exclusive_scan(v, s_tmp, &total);
        if (r < m) long_off[r] = running + excl;
        running += total;
    }
    if (threadIdx.x == 0) long_off[m] = running;
}

// Pass 5: tile t starts at long position t*TILE: tile_row[t] is the largest r
// with long_off[r] <= t*TILE, tile_nz[t] the offset inside that row.
template <int TILE>
__global__ __launch_bounds__(kBlock) void tile_search_kernel(int32_t m, int64_t num_tiles,
                                                             const int32_t *__restrict__ long_off,
                                                             int32_t *__restrict__ tile_row,
                                                             int32_t *__restrict__ tile_nz)
{
    const int64_t t = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (t > num_tiles) return;
    if (t == num_tiles) { tile_row[t] = m; tile_nz[t] = 0; return; }
    const int64_t pos = t * TILE;
    int32_t lo = 0, hi = m - 1;  // invariant: long_off[lo] <= pos, answer in [lo, hi]
    while (lo < hi) {
        const int32_t mid = lo + (hi - lo + 1) / 2;
        if (long_off[mid] <= pos) lo = mid; else hi = mid - 1;
    }
    tile_row[t] = lo;
    tile_nz[t] = (int32_t)(pos - long_off[lo]);
}


// The structure check works on tiles of kCheckTile consecutive entries.  tile_first[t] = the row
// that holds entry t * kCheckTile: the largest r in [0, nrows) with rowptr[r] <= t * kCheckTile
// (rows before it that start at the same entry are empty), for t = 0 .. num_tiles - 1, and
// tile_first[num_tiles] = nrows - 1.  One thread per tile; with a rowptr that is not monotone
// the result is some row id in [0, nrows) all the same.
constexpr int kCheckTile = kBlock * 8;
constexpr int kNumCheckFlags = 6;
__global__ __launch_bounds__(kBlock) void check_tile_rows_kernel(int32_t nrows, int64_t num_tiles,
                                                                 const int32_t *__restrict__ rowptr,
                                                                 int32_t *__restrict__ tile_first)
{
    const int64_t t = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (t > num_tiles) return;
    int32_t lo = 0, hi = nrows - 1;
    if (t == num_tiles) lo = hi;
    const int64_t j = t * kCheckTile;
    while (lo < hi) {
        const int32_t mid = lo + (hi - lo + 1) / 2;
        if (rowptr[mid] <= j) lo = mid; else hi = mid - 1;
    }
    tile_first[t] = lo;
}

// One pass over the structure, entry-parallel.  A workgroup takes a tile of kCheckTile entries:
// the rows that start inside the tile leave their id at their first entry's slot in LDS, a
// running maximum over the slots gives every entry its row (no search per entry), then each
// thread checks its entries.  flags must be 0 on entry:
//   flags[0] = 1 if rowptr decreases somewhere     flags[1] = 1 if a column is outside [0, ncols)
//   flags[2] = max |column - row| over the entries (the half bandwidth)
//   flags[3] = 1 if some row has a column smaller than its predecessor
//   flags[4] = 1 if rowptr[0] != 0 or rowptr[nrows] != nnz
//   flags[5] = number of entries followed, in their row, by the next column (runs of columns)
// With flags[0] or flags[4] set, flags[2], flags[3] and flags[5] are meaningless (every access stays in
// bounds all the same: row ids stay in [0, nrows), entry ids in [0, nnz) and LDS slots inside
// the tile).  nrows >= 1; tile_first comes from check_tile_rows_kernel.
__global__ __launch_bounds__(kBlock) void structure_check_kernel(int32_t nrows, int64_t ncols, int32_t nnz,
                                                                 const int32_t *__restrict__ rowptr,
                                                                 const int32_t *__restrict__ colidx,
                                                                 const int32_t *__restrict__ tile_first,
                                                                 int32_t *__restrict__ flags)
{
    constexpr int kPer = kCheckTile / kBlock;
    __shared__ int32_t s_row[kCheckTile + 1];
    __shared__ int32_t s_scan[kBlock];
    bool bad_row = false, bad_col = false, unsorted = false;
    int32_t best = 0, in_runs = 0;                     // in_runs: per wavefront (ballot counts)
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < nrows; i += stride)
        bad_row |= rowptr[i + 1] < rowptr[i];
    if (blockIdx.x == 0 && threadIdx.x == 0 && (rowptr[0] != 0 || rowptr[nrows] != nnz)) flags[4] = 1;
    const int tid = threadIdx.x;
    for (int64_t t = blockIdx.x; t * kCheckTile < nnz; t += gridDim.x) {
        const int32_t j0 = (int32_t)(t * kCheckTile);
        const int32_t j1 = (int32_t)((t * kCheckTile + kCheckTile < nnz) ? t * kCheckTile + kCheckTile : nnz);
        const int32_t first = tile_first[t], next = tile_first[t + 1];
        __syncthreads();                               // the previous tile's slots are no longer read
#pragma unroll
        for (int i = 0; i < kPer; ++i) s_row[i * kBlock + tid] = first;
        if (tid == 0) s_row[kCheckTile] = next;        // the row of entry j1, for the tile's last entry
        __syncthreads();
        // rows first+1 .. next start at an entry in (j0, j1] (when rowptr is monotone)
        for (int64_t r = (int64_t)first + 1 + tid; r <= next; r += kBlock) {
            const int32_t at = rowptr[r];
            if (at > j0 && at < j1) atomicMax(&s_row[at - j0], (int32_t)r);
        }
        __syncthreads();
        // running maximum over the slots: thread tid owns slots tid*kPer .. tid*kPer+kPer-1
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
            const int32_t j = j0 + pos;
            bool continues = false;
            if (j < j1) {
                const int32_t r = s_row[pos];
                const int32_t c = load_stream(colidx + j);
                bad_col |= (c < 0) | (c >= ncols);
                const int64_t d = (int64_t)c - r;
                const int64_t ad = d < 0 ? -d : d;
                best = max(best, (int32_t)(ad < INT32_MAX ? ad : INT32_MAX));
                // the next entry belongs to the same row: its slot (the tile's last entry: the next
                // tile's first row) holds the same row id
                const int32_t r_next = s_row[pos + 1 < j1 - j0 ? pos + 1 : kCheckTile];
                if (j + 1 < nnz && r_next == r) {
                    const int32_t c_next = colidx[j + 1];
                    unsorted |= c > c_next;
                    continues = c_next == c + 1;
                }
            }
            in_runs += (int32_t)__popcll(__ballot(continues));
        }
    }
    if (bad_row) flags[0] = 1;
    if (bad_col) flags[1] = 1;
    if (unsorted) flags[3] = 1;
    // one atomic per workgroup: atomics of many wavefronts on one address are served one by one
    best = wave_max_nonneg(best);
    __syncthreads();
    if (tid % kWave == 0) s_scan[tid / kWave] = best;
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < kWavesPerBlock; ++w) best = max(best, s_scan[w]);
        if (best > 0) atomicMax(&flags[2], best);
    }
    __syncthreads();
    if (tid % kWave == 0) s_scan[tid / kWave] = in_runs;
    __syncthreads();
    if (tid == 0) {
        int32_t total = 0;
        for (int w = 0; w < kWavesPerBlock; ++w) total += s_scan[w];
        if (total > 0) atomicAdd(&flags[5], total);
    }
}

// ---- column split of the rows above kWave entries ---------------------------
// When x is far larger than a level-2 cache, the rows of the last two bins are cut at the
// column-block boundaries b*W (b = 0..nb) into virtual rows, so that the gathers of one block
// stay cache resident while all rows' pieces in that block are processed.

// flag[0] = 1 if some split row has decreasing columns (the cut would then be wrong).
__global__ __launch_bounds__(kBlock) void split_sorted_kernel(int32_t S, const int32_t *__restrict__ split_rows,
                                                              const int32_t *__restrict__ rowptr,
                                                              const int32_t *__restrict__ colidx,
                                                              int32_t *__restrict__ flag)
{
    bool bad = false;
    for (int64_t r = blockIdx.x; r < S; r += gridDim.x) {
        const int32_t row = split_rows[r];
        const int64_t je = rowptr[row + 1];
        for (int64_t j = (int64_t)rowptr[row] + threadIdx.x; j + 1 < je; j += kBlock)
            bad |= colidx[j] > colidx[j + 1];
    }
    if (bad) flag[0] = 1;
}

// One workgroup of kCompactBlock threads: the rows of the last two bins (rows[0..count), in
// row_perm order) go, in that order, to split_rows if they have at most huge_row entries and to
// huge_rows otherwise; counts[0], counts[1] = how many of each.
__global__ __launch_bounds__(kCompactBlock) void split_rows_kernel(int32_t count, int32_t huge_row,
                                                                   const int32_t *__restrict__ rows,
                                                                   const int32_t *__restrict__ rowptr,
                                                                   int32_t *__restrict__ split_rows,
                                                                   int32_t *__restrict__ huge_rows,
                                                                   int32_t *__restrict__ counts)
{
    constexpr int kWaves = kCompactBlock / kWave;
    __shared__ int32_t s_wave[kWaves][2];
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    int32_t running[2] = {0, 0};
    for (int64_t base = 0; base < count; base += kCompactBlock) {
        const int64_t i = base + threadIdx.x;
        int32_t row = 0, cls = -1;
        if (i < count) {
            row = rows[i];
            cls = (rowptr[row + 1] - rowptr[row] > huge_row) ? 1 : 0;
        }
        const uint64_t m0 = __builtin_amdgcn_ballot_w64(cls == 0), m1 = __builtin_amdgcn_ballot_w64(cls == 1);
        if (lane == 0) { s_wave[wave][0] = __popcll(m0); s_wave[wave][1] = __popcll(m1); }
        __syncthreads();
        int32_t before[2] = {running[0], running[1]};
        for (int w = 0; w < kWaves; ++w) {
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const int32_t n = s_wave[w][k];
                if (w < wave) before[k] += n;
                running[k] += n;
            }
        }
        const uint64_t lower = (1ull << lane) - 1;
        if (cls == 0) split_rows[before[0] + __popcll(m0 & lower)] = row;
        if (cls == 1) huge_rows[before[1] + __popcll(m1 & lower)] = row;
        __syncthreads();
    }
    if (threadIdx.x < 2) counts[threadIdx.x] = running[threadIdx.x];
}

// cut[b*S + r] = first entry j of row split_rows[r] with colidx[j] >= b*W; cut[nb*S + r] = row end.
__global__ __launch_bounds__(kBlock) void split_cut_kernel(int32_t S, int32_t nb, int64_t W,
                                                           const int32_t *__restrict__ split_rows,
                                                           const int32_t *__restrict__ rowptr,
                                                           const int32_t *__restrict__ colidx,
                                                           int32_t *__restrict__ cut)
{
    const int64_t v = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= (int64_t)(nb + 1) * S) return;
    const int64_t b = v / S, r = v % S;
    const int32_t row = split_rows[r];
    int32_t lo = rowptr[row], hi = rowptr[row + 1];   // answer in [lo, hi]
    if (b < nb) {
        const int64_t target = b * W;
        while (lo < hi) {
            const int32_t mid = lo + (hi - lo) / 2;
            if ((int64_t)colidx[mid] < target) lo = mid + 1; else hi = mid;
        }
    } else {
        lo = hi;
    }
    cut[v] = lo;
}

// y[row] = alpha * sum_b vsum[b*S + r] + beta * y[row], blocks added in ascending order.
template <typename T>
__global__ __launch_bounds__(kBlock) void split_combine_kernel(int32_t S, int32_t nb,
                                                               const int32_t *__restrict__ split_rows,
                                                               const T *__restrict__ vsum,
                                                               T *__restrict__ y, T alpha, T beta)
{
    const int64_t r = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (r >= S) return;
    T s = T(0);
    for (int b = 0; b < nb; ++b) s += vsum[(int64_t)b * S + r];
    const int32_t row = split_rows[r];
    y[row] = (beta == T(0)) ? alpha * s : alpha * s + beta * y[row];
}

}  // namespace lapis
