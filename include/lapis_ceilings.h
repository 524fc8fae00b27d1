/*
 * lapis_ceilings.h - C ABI of the measurement kernels that bench.py times beside the products
 * (libceilings_mi355x.so; not part of the product library).  They measure what this GPU delivers
 * for the three access patterns the CSR kernels of Section 6.2's product are made of, so that a
 * kernel's time can be set against a measured ceiling as well as against the published HBM peak:
 *   read    one pass of 16-byte loads over a buffer (what streaming vals / colidx can reach);
 *   gather  8-byte gathers at random places of a table, indices streamed (the x gathers of a
 *           matrix with scattered columns: every gather that misses L2 moves a 128-byte line);
 *   rows    128-byte rows, 16 bytes per lane and 8 lanes per row, 16 rows in flight per lane,
 *           from a table that fits L2 or not (the rows of X an SpMM pulls through a CU's L1).
 * Every pointer is a DEVICE pointer the caller owns; nothing is allocated, copied or
 * synchronised; each call enqueues one kernel on hip_stream (a hipStream_t as void*).  The
 * kernels only read their inputs; d_sink (8 bytes at least) exists so that the loads cannot be
 * removed and is never written in practice.  Return value: 0, or 1 for an argument out of range
 * (null pointer, size not a multiple of 16, table length not a power of two, ...).
 */
#ifndef LAPIS_CEILINGS_H
#define LAPIS_CEILINGS_H
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

/* bytes: multiple of 16, d_buf 16-byte aligned; nontemporal != 0: loads carry the streaming hint */
int lapis_ceiling_read(const void *d_buf, int64_t bytes, int nontemporal, void *d_sink, void *hip_stream);

/* n gathers d_table[d_idx[i]]; indices outside [0, table_len) are read as index 0 */
int lapis_ceiling_gather(const double *d_table, int64_t table_len, const int32_t *d_idx, int64_t n, void *d_sink,
                         void *hip_stream);

/* num_waves wavefronts (one per workgroup) each read iters * 16 * 8 rows of 128 bytes from a table of
 * table_rows rows (a power of two); random != 0: the 8 rows of one load are unrelated, else consecutive.
 * Bytes delivered = num_waves * iters * 16 * 1024. */
int lapis_ceiling_rows(const double *d_table, int64_t table_rows, int32_t iters, int32_t num_waves, int random,
                       void *d_sink, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif
