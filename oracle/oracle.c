/*
 * CPU oracle for sparse x dense products and for the position cut.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call this file;
 * it is used by the tests, by the smoke check and by the benchmark's CPU
 * baseline leg.  It shares no code with the HIP kernels.
 *
 * The scheduled kernels of the paper compute, up to the order of the
 * floating-point additions, exactly what the unscheduled loop nests compute
 * (Section 5, "Parallelize": reordering only needs associativity), so the
 * oracle is the plain definition written out:
 *
 *   y(i)   = sum_j A(i,j) * x(j)          (Appendix, "SPMV on a CPU")
 *   C(i,k) = sum_j A(i,j) * B(j,k)        (Appendix, "SPMM on a CPU")
 *
 * over the coordinate hierarchy of a CSR matrix: a dense row level and a
 * compressed column level whose segment for row i is pos[i]..pos[i+1]
 * (Section 3).  Products and sums are taken in fp64 from the fp32 inputs.
 * Besides each result the functions return mag = sum_j |A(i,j) * x(j)|, the
 * scale of the admissible fp32 error of a row.
 *
 * BCSR (Section 1: a sparse matrix with dense inner dimensions) is the
 * four-level hierarchy (dense block row, compressed block column, dense row
 * in block, dense column in block) stored in lexicographic order (Section 3):
 * value (p, ii, ji) of block position p lives at vals[(p*bs + ii)*bs + ji].
 *
 * The position cut (Section 3, tiling the position space; Section 5,
 * "Split"; Section 6.2, coordinate recovery) splits positions 0..nnz into
 * tiles of `tile` positions.  tile_row[t] is the row that owns position
 * min(t*tile, nnz): the largest i with pos[i] <= that position.  The paper
 * finds it by binary search; the oracle instead walks the rows once, the way
 * the position loop of Section 3 advances i past row ends and empty rows.
 *
 * Further down: the same SpMV for fp64 operands (sums in extended precision), for a DCSR operand
 * (both levels compressed, Section 2), and MTTKRP A(i,j) = B(i,k,l) C(k,j) D(l,j) (Appendix, "MTTKRP
 * on a CPU") over a three-level compressed tensor with its two-level position cut.  All of them are
 * pinned by tests/test_oracle_pins.py; none is "parity unpinned".
 *
 * If `sel` is not NULL only the `nsel` listed rows are computed and outputs
 * are indexed by the position in the list (used to sample very large cases).
 * `threads` > 1 spreads rows over OpenMP threads; each row is still summed
 * serially, in storage order, by one thread.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int clamp_threads(int threads)
{
#ifdef _OPENMP
    if (threads < 1) threads = 1;
    int m = omp_get_max_threads();
    return threads > m ? m : threads;
#else
    (void)threads;
    return 1;
#endif
}

/* number of threads a call with this request would really use */
int oracle_threads(int threads) { return clamp_threads(threads); }

/* y(i) = A(i,j) * x(j), CSR.  y and mag have `rows` (or nsel) doubles; mag may be NULL. */
void oracle_spmv_csr(int64_t rows, const int32_t *pos, const int32_t *crd, const float *vals,
                     const float *x, double *y, double *mag, const int64_t *sel, int64_t nsel,
                     int threads)
{
    int64_t n = sel ? nsel : rows;
    threads = clamp_threads(threads);
#pragma omp parallel for schedule(dynamic, 1024) num_threads(threads)
    for (int64_t s = 0; s < n; ++s) {
        int64_t i = sel ? sel[s] : s;
        double acc = 0.0, m = 0.0;
        for (int64_t p = pos[i]; p < pos[i + 1]; ++p) {
            double t = (double)vals[p] * (double)x[crd[p]];
            acc += t;
            m += fabs(t);
        }
        y[s] = acc;
        if (mag) mag[s] = m;
    }
}

/* The same product for fp64 operands (the paper's own temporaries are Float64: appendix "SPMV on a
 * GPU").  Products and sums are formed in long double (x87 extended, 64-bit significand) and rounded
 * to double once, so that the reference carries ~2^-11 of the rounding error an fp64 kernel may have. */
void oracle_spmv_csr_f64(int64_t rows, const int32_t *pos, const int32_t *crd, const double *vals,
                         const double *x, double *y, double *mag, const int64_t *sel, int64_t nsel,
                         int threads)
{
    int64_t n = sel ? nsel : rows;
    threads = clamp_threads(threads);
#pragma omp parallel for schedule(dynamic, 1024) num_threads(threads)
    for (int64_t s = 0; s < n; ++s) {
        int64_t i = sel ? sel[s] : s;
        long double acc = 0.0L, m = 0.0L;
        for (int64_t p = pos[i]; p < pos[i + 1]; ++p) {
            long double t = (long double)vals[p] * (long double)x[crd[p]];
            acc += t;
            m += fabsl(t);
        }
        y[s] = (double)acc;
        if (mag) mag[s] = (double)m;
    }
}

/* C(i,k) = A(i,j) * B(j,k), CSR A, row-major B (ldb) and C (k doubles per row, packed). */
void oracle_spmm_csr(int64_t rows, int64_t k, const int32_t *pos, const int32_t *crd,
                     const float *vals, const float *B, int64_t ldb, double *C, double *mag,
                     const int64_t *sel, int64_t nsel, int threads)
{
    int64_t n = sel ? nsel : rows;
    threads = clamp_threads(threads);
#pragma omp parallel for schedule(dynamic, 256) num_threads(threads)
    for (int64_t s = 0; s < n; ++s) {
        int64_t i = sel ? sel[s] : s;
        double *c = C + s * k;
        double *m = mag ? mag + s * k : NULL;
        for (int64_t kk = 0; kk < k; ++kk) { c[kk] = 0.0; if (m) m[kk] = 0.0; }
        for (int64_t p = pos[i]; p < pos[i + 1]; ++p) {
            double a = (double)vals[p];
            const float *b = B + (int64_t)crd[p] * ldb;
            for (int64_t kk = 0; kk < k; ++kk) {
                double t = a * (double)b[kk];
                c[kk] += t;
                if (m) m[kk] += fabs(t);
            }
        }
    }
}

/* BCSR SpMV: brows block rows of bs x bs blocks; y, mag have brows*bs (or nsel*bs) doubles;
 * sel lists BLOCK rows. */
void oracle_spmv_bcsr(int64_t brows, int32_t bs, const int32_t *pos, const int32_t *crd,
                      const float *vals, const float *x, double *y, double *mag,
                      const int64_t *sel, int64_t nsel, int threads)
{
    int64_t n = sel ? nsel : brows;
    threads = clamp_threads(threads);
#pragma omp parallel for schedule(dynamic, 256) num_threads(threads)
    for (int64_t s = 0; s < n; ++s) {
        int64_t ib = sel ? sel[s] : s;
        for (int32_t ii = 0; ii < bs; ++ii) {
            double acc = 0.0, m = 0.0;
            for (int64_t p = pos[ib]; p < pos[ib + 1]; ++p) {
                int64_t jb = crd[p];
                for (int32_t ji = 0; ji < bs; ++ji) {
                    double t = (double)vals[(p * bs + ii) * bs + ji] * (double)x[jb * bs + ji];
                    acc += t;
                    m += fabs(t);
                }
            }
            y[s * bs + ii] = acc;
            if (mag) mag[s * bs + ii] = m;
        }
    }
}

/* BCSR SpMM: C((ib,ii),k) = sum over blocks p of row ib, ji: vals(p,ii,ji) * B((crd[p],ji),k). */
void oracle_spmm_bcsr(int64_t brows, int32_t bs, int64_t k, const int32_t *pos, const int32_t *crd,
                      const float *vals, const float *B, int64_t ldb, double *C, double *mag,
                      const int64_t *sel, int64_t nsel, int threads)
{
    int64_t n = sel ? nsel : brows;
    threads = clamp_threads(threads);
#pragma omp parallel for schedule(dynamic, 64) num_threads(threads)
    for (int64_t s = 0; s < n; ++s) {
        int64_t ib = sel ? sel[s] : s;
        for (int32_t ii = 0; ii < bs; ++ii) {
            double *c = C + (s * bs + ii) * k;
            double *m = mag ? mag + (s * bs + ii) * k : NULL;
            for (int64_t kk = 0; kk < k; ++kk) { c[kk] = 0.0; if (m) m[kk] = 0.0; }
            for (int64_t p = pos[ib]; p < pos[ib + 1]; ++p) {
                int64_t jb = crd[p];
                for (int32_t ji = 0; ji < bs; ++ji) {
                    double a = (double)vals[(p * bs + ii) * bs + ji];
                    const float *b = B + (jb * bs + ji) * ldb;
                    for (int64_t kk = 0; kk < k; ++kk) {
                        double t = a * (double)b[kk];
                        c[kk] += t;
                        if (m) m[kk] += fabs(t);
                    }
                }
            }
        }
    }
}

/* number of position tiles: ceil(nnz / tile) */
int64_t oracle_num_tiles(int64_t nnz, int64_t tile) { return nnz <= 0 ? 0 : (nnz + tile - 1) / tile; }

/*
 * Position cut: tile_row has oracle_num_tiles(nnz,tile)+1 entries.
 * One pass over the rows: i only ever advances (the tracking recurrence of
 * Section 6.2), stepping over a row when all of its positions, if it has any,
 * lie at or before the tile's first position.
 */
void oracle_partition(int64_t rows, int64_t nnz, const int32_t *pos, int64_t tile, int32_t *tile_row)
{
    int64_t ntiles = oracle_num_tiles(nnz, tile);
    int64_t i = 0;
    for (int64_t t = 0; t <= ntiles; ++t) {
        int64_t first = t * tile;
        if (first > nnz) first = nnz;
        while (i < rows && (int64_t)pos[i + 1] <= first) ++i;
        tile_row[t] = (int32_t)i;
    }
}

/*
 * MTTKRP on a three-level compressed tensor (appendix "MTTKRP on a GPU": A(i,j) = B(i,k,l) * C(k,j) * D(l,j)).
 * B is stored as a coordinate hierarchy (Section 3) with one level per mode: slice s (mode i; its
 * coordinate is crd_i[s], or s itself when crd_i is NULL = dense first level) owns fibers
 * pos_k[s] .. pos_k[s+1]; fiber q has coordinate crd_k[q] in mode k and owns leaf positions
 * pos_l[q] .. pos_l[q+1]; leaf p has coordinate crd_l[p] in mode l and value vals[p].
 * C is K x J (row stride ldc), D is L x J (row stride ldd).  out has J doubles per slice (or per
 * selected slice), indexed by SLICE, not by the slice's coordinate; mag likewise.
 */
void oracle_mttkrp_csf3(int64_t nslices, int64_t j, const int32_t *pos_k, const int32_t *crd_k,
                        const int32_t *pos_l, const int32_t *crd_l, const float *vals, const float *C,
                        int64_t ldc, const float *D, int64_t ldd, double *out, double *mag,
                        const int64_t *sel, int64_t nsel, int threads)
{
    int64_t n = sel ? nsel : nslices;
    threads = clamp_threads(threads);
#pragma omp parallel for schedule(dynamic, 64) num_threads(threads)
    for (int64_t t = 0; t < n; ++t) {
        int64_t s = sel ? sel[t] : t;
        double *a = out + t * j;
        double *m = mag ? mag + t * j : NULL;
        for (int64_t jj = 0; jj < j; ++jj) { a[jj] = 0.0; if (m) m[jj] = 0.0; }
        for (int64_t q = pos_k[s]; q < pos_k[s + 1]; ++q) {
            const float *c = C + (int64_t)crd_k[q] * ldc;
            for (int64_t p = pos_l[q]; p < pos_l[q + 1]; ++p) {
                const float *d = D + (int64_t)crd_l[p] * ldd;
                double v = (double)vals[p];
                for (int64_t jj = 0; jj < j; ++jj) {
                    double term = v * (double)c[jj] * (double)d[jj];
                    a[jj] += term;
                    if (m) m[jj] += fabs(term);
                }
            }
        }
    }
}

/*
 * Position cut of the leaf level of the three-level hierarchy (Section 3: a position loop keeps track of
 * every coordinate above the cut the same way).  For tile t with first leaf position min(t*tile, nnz):
 * tile_fiber[t] = largest q in [0, nfibers] with pos_l[q] <= that position, tile_slice[t] = largest s in
 * [0, nslices] with pos_k[s] <= tile_fiber[t].  Both tables have num_tiles + 1 entries.  One walk per level.
 */
void oracle_partition_csf3(int64_t nslices, int64_t nfibers, int64_t nnz, const int32_t *pos_k,
                           const int32_t *pos_l, int64_t tile, int32_t *tile_slice, int32_t *tile_fiber)
{
    int64_t ntiles = oracle_num_tiles(nnz, tile);
    int64_t q = 0, s = 0;
    for (int64_t t = 0; t <= ntiles; ++t) {
        int64_t first = t * tile;
        if (first > nnz) first = nnz;
        while (q < nfibers && (int64_t)pos_l[q + 1] <= first) ++q;
        while (s < nslices && (int64_t)pos_k[s + 1] <= q) ++s;
        tile_fiber[t] = (int32_t)q;
        tile_slice[t] = (int32_t)s;
    }
}

/* y(i) = A(i,j) * x(j) with A in DCSR: both levels compressed (Section 2 names DCSR among the concrete
 * forms of a coordinate hierarchy).  Stored row s has coordinate crd_i[s] (strictly increasing) and the
 * entries pos[s] .. pos[s+1]-1; rows that are not stored are zero.  y and mag have `rows` doubles. */
void oracle_spmv_dcsr(int64_t rows, int64_t nstored, const int32_t *crd_i, const int32_t *pos,
                      const int32_t *crd, const float *vals, const float *x, double *y, double *mag)
{
    for (int64_t i = 0; i < rows; ++i) { y[i] = 0.0; if (mag) mag[i] = 0.0; }
    for (int64_t s = 0; s < nstored; ++s) {
        double acc = 0.0, m = 0.0;
        for (int64_t p = pos[s]; p < pos[s + 1]; ++p) {
            double t = (double)vals[p] * (double)x[crd[p]];
            acc += t;
            m += fabs(t);
        }
        y[crd_i[s]] = acc;
        if (mag) mag[crd_i[s]] = m;
    }
}

/*
 * Structural validity of a CSR/BCSR index structure: pos[0]=0, pos monotone,
 * pos[rows]=nnz, 0 <= crd < cols.  Returns 0 if valid, else a code 1..4.
 */
int oracle_validate_csr(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd)
{
    if (pos[0] != 0) return 1;
    for (int64_t i = 0; i < rows; ++i)
        if (pos[i + 1] < pos[i]) return 2;
    if (pos[rows] != nnz) return 3;
    for (int64_t p = 0; p < nnz; ++p)
        if (crd[p] < 0 || crd[p] >= cols) return 4;
    return 0;
}

/*
 * The column-slab hierarchy of a CSR matrix and the SpMV evaluated over it.
 *
 * Section 8.6 obtains locality by tiling a dense-operand loop (split, then reorder); Section 3 allows
 * the position cut at any level of any coordinate hierarchy.  Here the column loop j is split by a fixed
 * slab width W, jo = j / W is moved outermost and the matrix is STORED in that order: a three-level
 * hierarchy (jo dense, i compressed, ji compressed).  Its leaf positions ("slots") are the stored
 * entries sorted by (jo, original position), i.e. a stable bucketing of the CSR positions by slab.
 * Every slab is padded with empty slots to a multiple of CH, so that chunks of CH slots never cross a
 * slab.  A "pair" is a maximal run of slots of one row inside one chunk; the product is evaluated as
 *     P(pair) = sum over the pair's slots of value * x(jo*W + ji)       (x of one slab at a time)
 *     y(i)    = sum of P over the pairs of row i
 * and the pairs of a row are listed by a CSR-like structure (qpos, qidx) in the order in which their
 * first slots occur in the original CSR.
 *
 *   svals[N], scol[N]: value and 15-bit in-slab column of each slot, bit 15 of scol = the slot is the
 *                      last of its pair; pad slots have value 0, column 0 and form pairs of their own
 *                      that no row lists.  scol is stored in slot order.  svals is stored in an order
 *                      permuted inside every chunk (a storage detail that lets CH / 8 lanes which own 8
 *                      consecutive slots each fetch them with contiguous 16-byte loads): when CH is a
 *                      multiple of 8, slot j of a chunk (lane l = j / 8, k = j % 8) sits at offset
 *                      (k / g) * (CH / 8 * g) + g * l + k % g of the chunk, g = values per 16 bytes
 *                      (4 for fp32: (k / 4) * (CH / 2) + 4 * l + k % 4; 2 for fp64:
 *                      (k / 2) * (CH / 4) + 2 * l + k % 2); otherwise at offset j.
 *   srow[N]:           row of each slot, -1 for pad slots (only needed while building);
 *   chunk_pair[N/CH + 1]: index of the pair that owns the first slot of each chunk; last = npairs;
 *   slab_chunk[S + 1]: first chunk of each slab; last = N/CH;
 *   qpos[rows + 1], qidx[nq]: the pairs of each row.
 * oracle_slab_count gives N, npairs and nq (array sizes); oracle_slab_build fills the arrays.
 * W must be at most 32768 (15 bits).
 */
static int64_t slab_layout(int64_t cols, int64_t nnz, const int32_t *crd, int64_t W, int64_t CH,
                           int64_t *base /* S + 1 */)
{
    int64_t S = (cols + W - 1) / W;
    for (int64_t s = 0; s <= S; ++s) base[s] = 0;
    for (int64_t p = 0; p < nnz; ++p) base[crd[p] / W + 1] += 1;           /* count of slab s at base[s+1] */
    for (int64_t s = 0; s < S; ++s) {
        int64_t padded = (base[s + 1] + CH - 1) / CH * CH;
        base[s + 1] = base[s] + padded;
    }
    return base[S];
}

/* Fills slot_row (row of each slot, -1 = pad) and slot_src (CSR position of each slot, -1 = pad). */
static void slab_slots(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd, int64_t W,
                       int64_t CH, const int64_t *base, int64_t N, int32_t *slot_row, int64_t *slot_src,
                       int64_t *fill /* S scratch */)
{
    int64_t S = (cols + W - 1) / W;
    (void)CH;
    for (int64_t j = 0; j < N; ++j) { slot_row[j] = -1; slot_src[j] = -1; }
    for (int64_t s = 0; s < S; ++s) fill[s] = 0;
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t p = pos[i]; p < pos[i + 1]; ++p) {
            int64_t s = crd[p] / W;
            int64_t j = base[s] + fill[s]++;
            slot_row[j] = (int32_t)i;
            slot_src[j] = p;
        }
    (void)nnz;
}

/* where the value of slot j is stored (see above); g = values per 16 bytes */
static int64_t slab_value_index_g(int64_t CH, int64_t j, int64_t g)
{
    if (CH % 8 != 0) return j;
    int64_t c = j / CH, o = j % CH, l = o / 8, k = o % 8;
    return c * CH + (k / g) * (CH / 8 * g) + g * l + k % g;
}
static int64_t slab_value_index(int64_t CH, int64_t j) { return slab_value_index_g(CH, j, 4); }

static int slab_is_start(const int32_t *slot_row, int64_t CH, int64_t j)
{
    return j % CH == 0 || slot_row[j] != slot_row[j - 1];
}

#include <stdlib.h>

/* sizes[0] = N (slots), sizes[1] = npairs, sizes[2] = nq (pairs listed by rows), sizes[3] = S.  Returns 0,
 * or -1 when memory runs out. */
int oracle_slab_count(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd, int64_t W,
                      int64_t CH, int64_t *sizes)
{
    int64_t S = (cols + W - 1) / W;
    int64_t *base = (int64_t *)malloc((size_t)(S + 1) * sizeof(int64_t));
    int64_t *fill = (int64_t *)malloc((size_t)(S + 1) * sizeof(int64_t));
    if (!base || !fill) { free(base); free(fill); return -1; }
    int64_t N = slab_layout(cols, nnz, crd, W, CH, base);
    int32_t *slot_row = (int32_t *)malloc((size_t)(N + 1) * sizeof(int32_t));
    int64_t *slot_src = (int64_t *)malloc((size_t)(N + 1) * sizeof(int64_t));
    if (!slot_row || !slot_src) { free(base); free(fill); free(slot_row); free(slot_src); return -1; }
    slab_slots(rows, cols, nnz, pos, crd, W, CH, base, N, slot_row, slot_src, fill);
    int64_t npairs = 0, nq = 0;
    for (int64_t j = 0; j < N; ++j)
        if (slab_is_start(slot_row, CH, j)) { ++npairs; if (slot_row[j] >= 0) ++nq; }
    sizes[0] = N; sizes[1] = npairs; sizes[2] = nq; sizes[3] = S;
    free(base); free(fill); free(slot_row); free(slot_src);
    return 0;
}

/* The structure for values of vbytes bytes each (4: float, 8: double); values are only moved. */
static int slab_build_any(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd,
                          const void *vals, int vbytes, int64_t W, int64_t CH, void *svals, uint16_t *scol,
                          int32_t *srow, int32_t *chunk_pair, int32_t *slab_chunk, int32_t *qpos, int32_t *qidx)
{
    int64_t S = (cols + W - 1) / W;
    int64_t g = 16 / vbytes;
    int64_t *base = (int64_t *)malloc((size_t)(S + 1) * sizeof(int64_t));
    int64_t *fill = (int64_t *)malloc((size_t)(S + 1) * sizeof(int64_t));
    if (!base || !fill) { free(base); free(fill); return -1; }
    int64_t N = slab_layout(cols, nnz, crd, W, CH, base);
    int64_t *slot_src = (int64_t *)malloc((size_t)(N + 1) * sizeof(int64_t));
    int32_t *pair_of = (int32_t *)malloc((size_t)(N + 1) * sizeof(int32_t));
    int64_t *slot_of = (int64_t *)malloc((size_t)(nnz + 1) * sizeof(int64_t));
    if (!slot_src || !pair_of || !slot_of) { free(base); free(fill); free(slot_src); free(pair_of); free(slot_of); return -1; }
    slab_slots(rows, cols, nnz, pos, crd, W, CH, base, N, srow, slot_src, fill);
    for (int64_t s = 0; s <= S; ++s) slab_chunk[s] = (int32_t)(base[s] / CH);
    /* slots: value, in-slab column; pairs numbered in slot order */
    int64_t npairs = 0;
    for (int64_t j = 0; j < N; ++j) {
        if (slab_is_start(srow, CH, j)) ++npairs;
        pair_of[j] = (int32_t)(npairs - 1);
        int64_t p = slot_src[j];
        int64_t at = slab_value_index_g(CH, j, g);
        if (vbytes == 4) ((float *)svals)[at] = p >= 0 ? ((const float *)vals)[p] : 0.0f;
        else ((double *)svals)[at] = p >= 0 ? ((const double *)vals)[p] : 0.0;
        scol[j] = p >= 0 ? (uint16_t)(crd[p] % W) : 0;
        if (p >= 0) slot_of[p] = j;
        if (j % CH == 0) chunk_pair[j / CH] = pair_of[j];
    }
    chunk_pair[N / CH] = (int32_t)npairs;
    for (int64_t j = 0; j < N; ++j)
        if (j == N - 1 || slab_is_start(srow, CH, j + 1)) scol[j] |= 0x8000u;
    /* the pairs of each row, in the order their first slots occur in the CSR */
    int64_t nq = 0;
    for (int64_t i = 0; i < rows; ++i) {
        qpos[i] = (int32_t)nq;
        for (int64_t p = pos[i]; p < pos[i + 1]; ++p) {
            int64_t j = slot_of[p];
            if (slab_is_start(srow, CH, j)) qidx[nq++] = pair_of[j];
        }
    }
    qpos[rows] = (int32_t)nq;
    free(base); free(fill); free(slot_src); free(pair_of); free(slot_of);
    return 0;
}

int oracle_slab_build(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd,
                      const float *vals, int64_t W, int64_t CH, float *svals, uint16_t *scol, int32_t *srow,
                      int32_t *chunk_pair, int32_t *slab_chunk, int32_t *qpos, int32_t *qidx)
{
    return slab_build_any(rows, cols, nnz, pos, crd, vals, 4, W, CH, svals, scol, srow, chunk_pair, slab_chunk, qpos,
                          qidx);
}

/* fp64 values (the paper's own value type, appendix "SPMV on a GPU"): same structure, 8-byte values */
int oracle_slab_build_f64(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd,
                          const double *vals, int64_t W, int64_t CH, double *svals, uint16_t *scol, int32_t *srow,
                          int32_t *chunk_pair, int32_t *slab_chunk, int32_t *qpos, int32_t *qidx)
{
    return slab_build_any(rows, cols, nnz, pos, crd, vals, 8, W, CH, svals, scol, srow, chunk_pair, slab_chunk, qpos,
                          qidx);
}

/* The SpMV evaluated over the structure, step by step as described above, in fp64: first P per pair, then
 * y per row (and mag = sum |value * x|).  P has npairs doubles (scratch).  Used to pin that the structure
 * represents the same matrix: its result must equal the CSR definition up to the order of the sums. */
void oracle_spmv_slab(int64_t rows, int64_t cols, int64_t N, int64_t W, int64_t CH, const float *svals,
                      const uint16_t *scol, const int32_t *slab_chunk, const int32_t *qpos, const int32_t *qidx,
                      const float *x, double *P, double *Pmag, double *y, double *mag)
{
    int64_t S = (cols + W - 1) / W;
    int64_t pair = 0;
    for (int64_t s = 0; s < S; ++s)
        for (int64_t j = (int64_t)slab_chunk[s] * CH; j < (int64_t)slab_chunk[s + 1] * CH; ++j) {
            double acc = 0.0, m = 0.0;
            for (;; ++j) {
                int64_t col = s * W + (scol[j] & 0x7fff);      /* pad slots: column 0 of the slab, value 0 */
                double t = (double)svals[slab_value_index(CH, j)] * (double)x[col];
                acc += t;
                m += fabs(t);
                if (scol[j] & 0x8000u) break;
            }
            P[pair] = acc;
            Pmag[pair] = m;
            ++pair;
        }
    (void)N;
    for (int64_t i = 0; i < rows; ++i) {
        double acc = 0.0, m = 0.0;
        for (int64_t q = qpos[i]; q < qpos[i + 1]; ++q) { acc += P[qidx[q]]; m += Pmag[qidx[q]]; }
        y[i] = acc;
        if (mag) mag[i] = m;
    }
}

/* The same for fp64 operands: products and sums in long double, P kept in long double, one rounding per row
 * (as oracle_spmv_csr_f64).  P and Pmag have npairs long doubles (scratch, allocated here). */
int oracle_spmv_slab_f64(int64_t rows, int64_t cols, int64_t npairs, int64_t W, int64_t CH, const double *svals,
                         const uint16_t *scol, const int32_t *slab_chunk, const int32_t *qpos,
                         const int32_t *qidx, const double *x, double *y, double *mag)
{
    int64_t S = (cols + W - 1) / W;
    long double *P = (long double *)malloc((size_t)(npairs + 1) * sizeof(long double));
    long double *Pmag = (long double *)malloc((size_t)(npairs + 1) * sizeof(long double));
    if (!P || !Pmag) { free(P); free(Pmag); return -1; }
    int64_t pair = 0;
    for (int64_t s = 0; s < S; ++s)
        for (int64_t j = (int64_t)slab_chunk[s] * CH; j < (int64_t)slab_chunk[s + 1] * CH; ++j) {
            long double acc = 0.0L, m = 0.0L;
            for (;; ++j) {
                int64_t col = s * W + (scol[j] & 0x7fff);
                long double t = (long double)svals[slab_value_index_g(CH, j, 2)] * (long double)x[col];
                acc += t;
                m += fabsl(t);
                if (scol[j] & 0x8000u) break;
            }
            P[pair] = acc;
            Pmag[pair] = m;
            ++pair;
        }
    for (int64_t i = 0; i < rows; ++i) {
        long double acc = 0.0L, m = 0.0L;
        for (int64_t q = qpos[i]; q < qpos[i + 1]; ++q) { acc += P[qidx[q]]; m += Pmag[qidx[q]]; }
        y[i] = (double)acc;
        if (mag) mag[i] = (double)m;
    }
    free(P); free(Pmag);
    return 0;
}
