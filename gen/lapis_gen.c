/*
 * Seeded synthetic input generators for the CSR SpMV / SpMM workloads.
 *
 * This file produces INPUTS only (sparsity structure, matrix values, dense
 * vectors).  It holds none of the method's arithmetic: no products, no row
 * sums, no partitioning.  Both the CPU oracle's tests and the GPU library's
 * tests feed on the arrays written here.
 *
 * Randomness is counter based: every drawn number is a pure function of
 * (seed, stream, index), so the arrays do not depend on thread count, on the
 * order of generation or on any library's generator.  The mixing function is
 * the SplitMix64 output permutation (Steele, Lea, Flood 2014) applied twice.
 *
 * Streams used by the Python layer: 0 structure, 1 matrix values, 2 x / X,
 * 3 y0 / Y0.
 *
 * The matrices stand in for the SuiteSparse / Galeri matrices of the paper's
 * Table 3 (Section 6.2), which are not available offline.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static inline uint64_t mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

/* 64 pseudo-random bits for (seed, stream, index). */
uint64_t lapis_gen_bits(uint64_t seed, uint64_t stream, uint64_t index)
{
    uint64_t h = mix64(seed + 0x9E3779B97F4A7C15ULL * (stream + 1));
    return mix64(h + 0x9E3779B97F4A7C15ULL * (index + 1));
}

/* Uniform double in [0,1) with 53 random bits. */
static inline double u01(uint64_t seed, uint64_t stream, uint64_t index)
{
    return (double)(lapis_gen_bits(seed, stream, index) >> 11) * 0x1.0p-53;
}

void lapis_gen_uniform_f64(uint64_t seed, uint64_t stream, double lo, double hi,
                           double *out, int64_t n)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        out[i] = lo + (hi - lo) * u01(seed, stream, (uint64_t)i);
}

/* Uniform float in [lo,hi): the double draw is rounded to float and, if that
 * rounding lands on hi, moved to the largest float below hi. */
void lapis_gen_uniform_f32(uint64_t seed, uint64_t stream, double lo, double hi,
                           float *out, int64_t n)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        float v = (float)(lo + (hi - lo) * u01(seed, stream, (uint64_t)i));
        if (v >= (float)hi) v = nextafterf((float)hi, (float)lo);
        out[i] = v;
    }
}

/* Standard normal by Box-Muller; element i consumes indices 2i and 2i+1. */
void lapis_gen_normal_f64(uint64_t seed, uint64_t stream, double *out, int64_t n)
{
    const double two_pi = 6.283185307179586476925286766559;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double u1 = ((double)(lapis_gen_bits(seed, stream, 2 * (uint64_t)i) >> 11) + 1.0) * 0x1.0p-53;
        double u2 = u01(seed, stream, 2 * (uint64_t)i + 1);
        out[i] = sqrt(-2.0 * log(u1)) * cos(two_pi * u2);
    }
}

/* ------------------------------------------------------------------------
 * 2D 5-point Poisson stencil, Dirichlet boundary (neighbours outside the grid
 * are dropped).  Row = i*ny_cols + j for grid point (i, j) with j fastest;
 * entries in ascending column order; diagonal 4, off-diagonals -1.
 * rowptr has nx*ny+1 entries; returns nnz.  Pass colidx = vals = NULL to count.
 * ---------------------------------------------------------------------- */
int64_t lapis_gen_poisson2d(int64_t nx, int64_t ny, int32_t *rowptr,
                            int32_t *colidx, double *vals)
{
    int64_t e = 0;
    for (int64_t i = 0; i < nx; ++i) {
        for (int64_t j = 0; j < ny; ++j) {
            int64_t r = i * ny + j;
            rowptr[r] = (int32_t)e;
            const int64_t di[5] = {-1, 0, 0, 0, 1};
            const int64_t dj[5] = {0, -1, 0, 1, 0};
            for (int t = 0; t < 5; ++t) {
                int64_t a = i + di[t], b = j + dj[t];
                if (a < 0 || a >= nx || b < 0 || b >= ny) continue;
                if (colidx) {
                    colidx[e] = (int32_t)(a * ny + b);
                    vals[e] = (t == 2) ? 4.0 : -1.0;
                }
                ++e;
            }
        }
    }
    rowptr[nx * ny] = (int32_t)e;
    return e;
}

/* ------------------------------------------------------------------------
 * 3D 27-point stencil on an nx*ny*nz grid, neighbours outside the grid are
 * dropped.  Row = (z*ny + y)*nx + x.  Entries in lexicographic (dz,dy,dx)
 * order, which is ascending column order.  One independent draw per stored
 * entry, indexed by the entry's position e in CSR order (stream 1):
 * off-diagonal = -1 + u (in [-1,0)), diagonal = 26 + u (in [26,27)).
 * Step 1: lapis_gen_stencil27_rowptr fills rowptr and returns nnz.
 * Step 2: lapis_gen_stencil27_fill fills colidx and vals.
 * ---------------------------------------------------------------------- */
static inline int span(int64_t c, int64_t n) /* neighbours of c inside [0,n) among c-1,c,c+1 */
{
    return 1 + (c > 0) + (c + 1 < n);
}

int64_t lapis_gen_stencil27_rowptr(int64_t nx, int64_t ny, int64_t nz, int32_t *rowptr)
{
    int64_t e = 0, r = 0;
    for (int64_t z = 0; z < nz; ++z)
        for (int64_t y = 0; y < ny; ++y)
            for (int64_t x = 0; x < nx; ++x) {
                rowptr[r++] = (int32_t)e;
                e += (int64_t)span(x, nx) * span(y, ny) * span(z, nz);
            }
    rowptr[r] = (int32_t)e;
    return e;
}

void lapis_gen_stencil27_fill(int64_t nx, int64_t ny, int64_t nz, uint64_t seed,
                              const int32_t *rowptr, int32_t *colidx, double *vals)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < nx * ny * nz; ++r) {
        int64_t x = r % nx, y = (r / nx) % ny, z = r / (nx * ny);
        int64_t e = rowptr[r];
        for (int64_t dz = -1; dz <= 1; ++dz) {
            if (z + dz < 0 || z + dz >= nz) continue;
            for (int64_t dy = -1; dy <= 1; ++dy) {
                if (y + dy < 0 || y + dy >= ny) continue;
                for (int64_t dx = -1; dx <= 1; ++dx) {
                    if (x + dx < 0 || x + dx >= nx) continue;
                    int64_t c = ((z + dz) * ny + (y + dy)) * nx + (x + dx);
                    double u = u01(seed, 1, (uint64_t)e);
                    colidx[e] = (int32_t)c;
                    vals[e] = (c == r) ? 26.0 + u : -1.0 + u;
                    ++e;
                }
            }
        }
    }
}

/* ------------------------------------------------------------------------
 * Fixed row length: every row holds exactly per_row distinct columns drawn
 * uniformly from [0, ncols) by rejection (a repeated column is redrawn), then
 * sorted ascending.  Draw t of row i uses (stream 0, index i*1024 + t).
 * Requires per_row <= ncols and per_row <= 64.  Returns 0, or -1 on bad
 * arguments or if a row needed more than 1024 draws.
 * ---------------------------------------------------------------------- */
int lapis_gen_fixed_rows(int64_t nrows, int64_t ncols, int per_row, uint64_t seed,
                         int32_t *rowptr, int32_t *colidx)
{
    if (per_row < 0 || per_row > 64 || per_row > ncols) return -1;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t i = 0; i < nrows; ++i) {
        int32_t c[64];
        int have = 0;
        uint64_t t = 0;
        while (have < per_row && t < 1024) {
            uint64_t bits = lapis_gen_bits(seed, 0, (uint64_t)i * 1024 + t++);
            /* multiply-shift maps 64 bits to [0, ncols) without modulo bias that matters here */
            int32_t col = (int32_t)(((unsigned __int128)bits * (uint64_t)ncols) >> 64);
            int dup = 0;
            for (int q = 0; q < have; ++q) dup |= (c[q] == col);
            if (!dup) c[have++] = col;
        }
        if (have < per_row) { bad = 1; continue; }
        for (int a = 1; a < per_row; ++a) { /* insertion sort */
            int32_t v = c[a];
            int b = a - 1;
            while (b >= 0 && c[b] > v) { c[b + 1] = c[b]; --b; }
            c[b + 1] = v;
        }
        rowptr[i] = (int32_t)(i * per_row);
        memcpy(colidx + i * per_row, c, sizeof(int32_t) * (size_t)per_row);
    }
    rowptr[nrows] = (int32_t)(nrows * per_row);
    return bad ? -1 : 0;
}

/* ------------------------------------------------------------------------
 * Power-law row lengths: L in {1..cap} with P(L = l) = l^-s / zeta(s) for
 * l < cap and all remaining tail mass on L = cap (clipping, not truncation
 * with renormalisation).  Inverse CDF on one uniform draw per row
 * (stream 0, index i).  Writes len[nrows]; returns 0 or -1.
 * ---------------------------------------------------------------------- */
int lapis_gen_zipf_lengths(int64_t nrows, double s, int64_t cap, uint64_t seed, int32_t *len)
{
    if (s <= 1.0 || cap < 1 || cap > 0x7fffffff) return -1;
    double *cdf = (double *)malloc(sizeof(double) * (size_t)cap); /* cdf[l-1] = P(L <= l), unnormalised, l < cap */
    if (!cdf) return -1;
    double acc = 0.0;
    for (int64_t l = 1; l < cap; ++l) { acc += pow((double)l, -s); cdf[l - 1] = acc; }
    /* tail sum_{l >= cap} l^-s by Euler-Maclaurin */
    double c = (double)cap;
    double tail = pow(c, 1.0 - s) / (s - 1.0) + 0.5 * pow(c, -s) + s * pow(c, -s - 1.0) / 12.0
                - s * (s + 1.0) * (s + 2.0) * pow(c, -s - 3.0) / 720.0;
    double zeta = acc + tail;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nrows; ++i) {
        double target = u01(seed, 0, (uint64_t)i) * zeta;
        /* smallest l with cdf[l-1] > target; none below cap -> cap */
        int64_t lo = 0, hi = cap - 1; /* search over indices [0, cap-1) */
        while (lo < hi) {
            int64_t mid = (lo + hi) >> 1;
            if (cdf[mid] > target) hi = mid; else lo = mid + 1;
        }
        len[i] = (int32_t)(lo + 1); /* lo == cap-1 means no index qualified -> L = cap */
    }
    free(cdf);
    return 0;
}

/* Exclusive prefix sum of len into rowptr[nrows+1]; returns the total, or -1
 * if it does not fit in int32. */
int64_t lapis_gen_rowptr_from_lengths(int64_t nrows, const int32_t *len, int32_t *rowptr)
{
    int64_t e = 0;
    for (int64_t i = 0; i < nrows; ++i) {
        rowptr[i] = (int32_t)e;
        e += len[i];
        if (e > 0x7fffffff) return -1;
    }
    rowptr[nrows] = (int32_t)e;
    return e;
}

/* ------------------------------------------------------------------------
 * Distinct sorted columns for arbitrary row lengths L <= ncols by stratified
 * jitter: entry j of a row of length L falls in stratum
 * [floor(j*ncols/L), floor((j+1)*ncols/L)) at a uniform position
 * (stream 0, index = 2^40 + entry position).  Strata are disjoint and
 * ascending, so the row is sorted and duplicate free by construction.
 * ---------------------------------------------------------------------- */
int lapis_gen_stratified_cols(int64_t nrows, int64_t ncols, const int32_t *rowptr,
                              uint64_t seed, int32_t *colidx)
{
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1024) reduction(| : bad)
    for (int64_t i = 0; i < nrows; ++i) {
        int64_t b = rowptr[i], L = rowptr[i + 1] - b;
        if (L > ncols) { bad = 1; continue; }
        for (int64_t j = 0; j < L; ++j) {
            int64_t s0 = (int64_t)(((unsigned __int128)j * (uint64_t)ncols) / (uint64_t)L);
            int64_t s1 = (int64_t)(((unsigned __int128)(j + 1) * (uint64_t)ncols) / (uint64_t)L);
            uint64_t bits = lapis_gen_bits(seed, 0, (1ULL << 40) + (uint64_t)(b + j));
            int64_t off = (int64_t)(((unsigned __int128)bits * (uint64_t)(s1 - s0)) >> 64);
            colidx[b + j] = (int32_t)(s0 + off);
        }
    }
    return bad ? -1 : 0;
}

/* ------------------------------------------------------------------------
 * Block stencil: 27-point stencil on an nx*ny*nz grid with `dof` unknowns per
 * grid point, every pair of unknowns of neighbouring points coupled (3-D
 * elasticity on a regular grid has this shape: 81 entries per interior row for
 * dof = 3).  Row = node*dof + d, node = (z*ny + y)*nx + x; columns ascending.
 * One draw per stored entry (stream 1, index = CSR position): diagonal
 * 27*dof + u, others -1 + u.
 * ---------------------------------------------------------------------- */
int64_t lapis_gen_block_stencil_rowptr(int64_t nx, int64_t ny, int64_t nz, int64_t dof, int32_t *rowptr)
{
    int64_t e = 0, r = 0;
    for (int64_t z = 0; z < nz; ++z)
        for (int64_t y = 0; y < ny; ++y)
            for (int64_t x = 0; x < nx; ++x) {
                int64_t nb = (int64_t)span(x, nx) * span(y, ny) * span(z, nz);
                for (int64_t d = 0; d < dof; ++d) { rowptr[r++] = (int32_t)e; e += nb * dof; }
            }
    rowptr[r] = (int32_t)e;
    return e;
}

void lapis_gen_block_stencil_fill(int64_t nx, int64_t ny, int64_t nz, int64_t dof, uint64_t seed,
                                  const int32_t *rowptr, int32_t *colidx, double *vals)
{
#pragma omp parallel for schedule(static)
    for (int64_t node = 0; node < nx * ny * nz; ++node) {
        int64_t x = node % nx, y = (node / nx) % ny, z = node / (nx * ny);
        for (int64_t d = 0; d < dof; ++d) {
            int64_t r = node * dof + d;
            int64_t e = rowptr[r];
            for (int64_t dz = -1; dz <= 1; ++dz) {
                if (z + dz < 0 || z + dz >= nz) continue;
                for (int64_t dy = -1; dy <= 1; ++dy) {
                    if (y + dy < 0 || y + dy >= ny) continue;
                    for (int64_t dx = -1; dx <= 1; ++dx) {
                        if (x + dx < 0 || x + dx >= nx) continue;
                        int64_t nbr = ((z + dz) * ny + (y + dy)) * nx + (x + dx);
                        for (int64_t q = 0; q < dof; ++q) {
                            int64_t c = nbr * dof + q;
                            double u = u01(seed, 1, (uint64_t)e);
                            colidx[e] = (int32_t)c;
                            vals[e] = (c == r) ? 27.0 * (double)dof + u : -1.0 + u;
                            ++e;
                        }
                    }
                }
            }
        }
    }
}

/* ------------------------------------------------------------------------
 * Row lengths with a prescribed mean and maximum: L = clamp(round(mean * g), 1,
 * max_len) with g a Gamma(4, 1/4) variate (mean 1, built from four uniform
 * draws: -log(u1 u2 u3 u4)/4; stream 0, indices 4i..4i+3); row 0 is set to
 * max_len so the maximum is attained.
 * ---------------------------------------------------------------------- */
void lapis_gen_gamma_lengths(int64_t nrows, double mean, int64_t max_len, uint64_t seed, int32_t *len)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nrows; ++i) {
        double p = 1.0;
        for (int q = 0; q < 4; ++q)
            p *= ((double)(lapis_gen_bits(seed, 0, 4 * (uint64_t)i + q) >> 11) + 1.0) * 0x1.0p-53;
        double L = floor(mean * (-log(p) / 4.0) + 0.5);
        if (L < 1.0) L = 1.0;
        if (L > (double)max_len) L = (double)max_len;
        len[i] = (int32_t)L;
    }
    if (nrows > 0) len[0] = (int32_t)max_len;
}

/* ------------------------------------------------------------------------
 * Banded distinct sorted columns: the L columns of row i are spread by
 * stratified jitter over the window of width min(ncols, band_factor * L)
 * centred on the diagonal (shifted to stay inside [0, ncols)).
 * Draw index = 2^41 + entry position (stream 0).
 * ---------------------------------------------------------------------- */
int lapis_gen_banded_cols(int64_t nrows, int64_t ncols, const int32_t *rowptr, int64_t band_factor,
                          uint64_t seed, int32_t *colidx)
{
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1024) reduction(| : bad)
    for (int64_t i = 0; i < nrows; ++i) {
        int64_t b = rowptr[i], L = rowptr[i + 1] - b;
        if (L > ncols) { bad = 1; continue; }
        int64_t width = band_factor * L;
        if (width > ncols) width = ncols;
        if (width < L) width = L;
        int64_t centre = (int64_t)(((unsigned __int128)i * (uint64_t)ncols) / (uint64_t)(nrows > 0 ? nrows : 1));
        int64_t lo = centre - width / 2;
        if (lo < 0) lo = 0;
        if (lo + width > ncols) lo = ncols - width;
        for (int64_t j = 0; j < L; ++j) {
            int64_t s0 = (int64_t)(((unsigned __int128)j * (uint64_t)width) / (uint64_t)L);
            int64_t s1 = (int64_t)(((unsigned __int128)(j + 1) * (uint64_t)width) / (uint64_t)L);
            uint64_t bits = lapis_gen_bits(seed, 0, (1ULL << 41) + (uint64_t)(b + j));
            int64_t off = (int64_t)(((unsigned __int128)bits * (uint64_t)(s1 - s0)) >> 64);
            colidx[b + j] = (int32_t)(lo + s0 + off);
        }
    }
    return bad ? -1 : 0;
}
