/*
 * Seeded synthetic input generators (host C, OpenMP).
 *
 * This file produces inputs only: sparsity patterns, values and dense
 * operands.  It contains none of the method's arithmetic (no products, no
 * reductions, no position cut), so that the oracle and the HIP path can both
 * be fed from it without sharing any logic with each other.
 *
 * Random numbers are counter based: every draw is splitmix64's output
 * function applied to a key built from (seed, stream, index), so any element
 * can be produced independently and in parallel and the bytes do not depend
 * on the thread count.
 *
 * Real values are  lo + (hi-lo) * m * 2^-24  with a 24-bit integer m, i.e.
 * uniform on a grid that fp32 represents exactly for the ranges used here
 * ([-1,1) and [0.5,1.5)).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static inline uint64_t mix64(uint64_t z)
{
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

static inline uint64_t draw(uint64_t seed, uint64_t stream, uint64_t index)
{
    return mix64(mix64(seed ^ (stream * 0xD1342543DE82EF95ull)) ^ (index * 0xA0761D6478BD642Full));
}

static inline float unit24(uint64_t r, float lo, float hi)
{
    /* 24 random bits -> exactly representable fp32 in [lo, hi) */
    return lo + (hi - lo) * ((float)(r >> 40) * (1.0f / 16777216.0f));
}

/* out[i] = uniform in [lo,hi), i in [0,n) */
void wl_fill_uniform(float *out, int64_t n, uint64_t seed, uint64_t stream, float lo, float hi)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        out[i] = unit24(draw(seed, stream, (uint64_t)i), lo, hi);
}

/*
 * Row lengths from a truncated Zipf law: P(len = k) proportional to k^-alpha
 * for k in [kmin, kmax], sampled by inverting the cumulative distribution.
 * Returns 0, or -1 on allocation failure / bad arguments.
 */
int wl_zipf_lengths(int32_t *len, int64_t rows, double alpha, int32_t kmin, int32_t kmax,
                    uint64_t seed, uint64_t stream)
{
    if (kmin < 0 || kmax < kmin) return -1;
    int64_t m = (int64_t)kmax - kmin + 1;
    double *cdf = (double *)malloc((size_t)m * sizeof(double));
    if (!cdf) return -1;
    double acc = 0.0;
    for (int64_t k = 0; k < m; ++k) {
        acc += pow((double)(kmin + k), -alpha);
        cdf[k] = acc;
    }
    const double total = acc;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        uint64_t bits = draw(seed, stream, (uint64_t)r) >> 11;      /* 53 bits */
        double u = (double)bits * (1.0 / 9007199254740992.0) * total; /* [0,total) */
        int64_t lo = 0, hi = m - 1;                                  /* first k with cdf[k] > u */
        while (lo < hi) {
            int64_t mid = (lo + hi) >> 1;
            if (cdf[mid] > u) hi = mid; else lo = mid + 1;
        }
        len[r] = (int32_t)(kmin + lo);
    }
    free(cdf);
    return 0;
}

static int cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/*
 * For every row r, fill crd[pos[r] .. pos[r+1]) with pos[r+1]-pos[r] DISTINCT
 * column indices drawn uniformly from [0, cols), sorted ascending.
 * Each row has its own random stream keyed by (seed, stream, r), so the
 * result does not depend on scheduling.  A row longer than cols is an error.
 * Returns 0 or -1.
 */
int wl_csr_columns(const int32_t *pos, int64_t rows, int64_t cols, uint64_t seed, uint64_t stream,
                   int32_t *crd)
{
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 256) reduction(| : bad)
    for (int64_t r = 0; r < rows; ++r) {
        int64_t n = (int64_t)pos[r + 1] - pos[r];
        if (n <= 0) continue;
        if (n > cols) { bad = 1; continue; }
        int32_t *c = crd + pos[r];
        uint64_t key = mix64(seed ^ (stream * 0xD1342543DE82EF95ull)) ^ ((uint64_t)r * 0xA0761D6478BD642Full);
        uint64_t ctr = 0;
        if (n == cols) { for (int64_t k = 0; k < n; ++k) c[k] = (int32_t)k; continue; }
        if (n <= 48) {
            /* sorted insertion with duplicate rejection */
            int64_t have = 0;
            while (have < n) {
                int32_t v = (int32_t)(mix64(key + (ctr++) * 0x9E3779B97F4A7C15ull) % (uint64_t)cols);
                int64_t i = have;
                while (i > 0 && c[i - 1] > v) --i;
                if (i > 0 && c[i - 1] == v) continue;
                memmove(c + i + 1, c + i, (size_t)(have - i) * sizeof(int32_t));
                c[i] = v;
                ++have;
            }
        } else {
            /* draw the deficit, sort, drop duplicates, repeat */
            int64_t have = 0;
            while (have < n) {
                for (int64_t k = have; k < n; ++k)
                    c[k] = (int32_t)(mix64(key + (ctr++) * 0x9E3779B97F4A7C15ull) % (uint64_t)cols);
                qsort(c, (size_t)n, sizeof(int32_t), cmp_i32);
                int64_t w = 1;
                for (int64_t k = 1; k < n; ++k)
                    if (c[k] != c[w - 1]) c[w++] = c[k];
                have = w;
            }
        }
    }
    return bad ? -1 : 0;
}

/*
 * 27-point stencil on an n x n x n grid, faces clipped (no wrap).
 * Row index i = x + n*(y + n*z); neighbours visited in (dz,dy,dx) order so the
 * columns of a row ascend.  Off-diagonal values uniform in [0.5,1.5) keyed by
 * the position index, diagonal exactly 27.
 * pos has n^3+1 entries; crd/vals have (3n-2)^3 entries (callers size them
 * with wl_stencil27_nnz).  pos entries are int32: n <= 160 keeps nnz < 2^31.
 */
int64_t wl_stencil27_nnz(int64_t n) { return n <= 0 ? 0 : (n == 1 ? 1 : (3 * n - 2) * (3 * n - 2) * (3 * n - 2)); }

static inline int span(int64_t c, int64_t n) { return 1 + (c > 0) + (c < n - 1); }

int wl_stencil27(int64_t n, uint64_t seed, uint64_t stream, int32_t *pos, int32_t *crd, float *vals)
{
    if (n <= 0 || wl_stencil27_nnz(n) > 2147483647ll) return -1;
    /* row starts: rows of one z-plane have lengths sx*sy*sz; prefix-sum exactly, serially per plane */
    int64_t p = 0;
    for (int64_t z = 0; z < n; ++z)
        for (int64_t y = 0; y < n; ++y)
            for (int64_t x = 0; x < n; ++x) {
                pos[x + n * (y + n * z)] = (int32_t)p;
                p += (int64_t)span(x, n) * span(y, n) * span(z, n);
            }
    pos[n * n * n] = (int32_t)p;
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t z = 0; z < n; ++z)
        for (int64_t y = 0; y < n; ++y)
            for (int64_t x = 0; x < n; ++x) {
                int64_t i = x + n * (y + n * z);
                int64_t q = pos[i];
                for (int dz = -1; dz <= 1; ++dz) {
                    int64_t zz = z + dz; if (zz < 0 || zz >= n) continue;
                    for (int dy = -1; dy <= 1; ++dy) {
                        int64_t yy = y + dy; if (yy < 0 || yy >= n) continue;
                        for (int dx = -1; dx <= 1; ++dx) {
                            int64_t xx = x + dx; if (xx < 0 || xx >= n) continue;
                            int64_t j = xx + n * (yy + n * zz);
                            crd[q] = (int32_t)j;
                            vals[q] = (j == i) ? 27.0f : unit24(draw(seed, stream, (uint64_t)q), 0.5f, 1.5f);
                            ++q;
                        }
                    }
                }
            }
    return 0;
}
