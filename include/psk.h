/*
 * psk -- position-space sparse x dense kernels for AMD MI355X (gfx950).
 *
 * C ABI of the library.  The operations are the two statements of the paper's
 * appendix, scheduled by hand the way its GPU schedules do it (fuse the row
 * and column loops, move the fused loop into the position space of A, split
 * it into equal tiles -- appendix "SPMV on a GPU", "SPMM on a GPU"; Sections
 * 3 and 5):
 *
 *     y(i)   = A(i,j) * x(j)            SpMV
 *     C(i,k) = A(i,j) * B(j,k)          SpMM, dense row-major B and C
 *
 * A is CSR (Section 3: dense row level, compressed column level; row i owns
 * positions pos[i] .. pos[i+1] of crd/vals) or BCSR (Section 1: the same with
 * a dense bs x bs block per stored position, row-major inside the block,
 * vals[(p*bs + ii)*bs + ji]).
 *
 * Further down, the same cut on other operands and statements: A in DCSR (both
 * levels compressed), fp64 values, the MTTKRP statement of the appendix on a
 * three-level compressed tensor, a variant that divides the position space
 * into a fixed number of parts, and the baselines/ablations of Section 8.
 * Each entry point states what differs from the conventions below.
 *
 * Conventions for every entry point
 *  - Every pointer is a DEVICE pointer owned by the caller.  The library does
 *    not allocate, free or keep any of them.  Scratch memory is passed in as
 *    `workspace` (size from psk_workspace_bytes; 256-byte aligned).
 *  - `stream` is a hipStream_t passed as void* (NULL = the null stream).  A
 *    call only enqueues work on that stream and returns; it never
 *    synchronises.  Calls that share a workspace must be stream-ordered.
 *  - Index arrays are int32, values and dense operands fp32; products and sums
 *    are fp32 on the device (carries between tiles are combined in fp64).
 *    psk_spmv_csr_f64, psk_slab_build_csr_f64 and psk_spmv_slab_f64 are all fp64.
 *  - Outputs are assigned, not accumulated: rows without stored entries
 *    become +0.0f.  Inputs and outputs must not overlap.
 *  - Results are run-to-run deterministic: every y(i) / C(i,k) has one writer
 *    and a fixed summation order for a given tile size (the one exception is
 *    the baseline psk_spmv_csr_atomics).
 *  - Only psk_analyze_csr, psk_suggest_schedule_csr and psk_validate_csr synchronise the
 *    stream (they read one number back); they say so.
 *  - Preconditions that are NOT checked on the device (caller's contract):
 *    pos[0] = 0, pos non-decreasing, pos[rows] = nnz, 0 <= crd[p] < cols.
 *    Columns inside a row need not be sorted or distinct (duplicates add up).
 *  - Return value: PSK_OK or an error code; nothing is enqueued on error
 *    (except PSK_ERR_HIP, which reports a failed launch).  No call aborts.
 *  - Sizes: 0 <= rows, cols; 0 <= nnz <= 2^31-1.  Empty problems are valid.
 *  - `tile` is the position-tile size (the split factor of the position
 *    loop, Section 5 "Split"): the number of stored positions per workgroup.
 *    0 selects the library default; otherwise it must be one of the sizes
 *    listed with each operation, else PSK_ERR_TILE.
 *  - `phases` selects which steps run (bit mask, PSK_PHASE_ALL for a
 *    complete product).  PSK_PHASE_PARTITION writes the tile->row table into
 *    the workspace; it depends only on (pos, nnz, tile), so a caller that
 *    multiplies by the same A again may leave it out.  PSK_PHASE_MAIN streams
 *    the tiles; PSK_PHASE_FIXUP adds the carries of rows that span tiles.
 *    A call without PSK_PHASE_FIXUP leaves those rows incomplete (useful
 *    only for measuring the steps separately).
 */
#ifndef PSK_H
#define PSK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PSK_OK = 0,
    PSK_ERR_NULL = 1,        /* a required pointer is NULL */
    PSK_ERR_SIZE = 2,        /* negative size, nnz > 2^31-1, k <= 0, bad leading dimension, bad block size */
    PSK_ERR_TILE = 3,        /* tile size not supported by this operation */
    PSK_ERR_WORKSPACE = 4,   /* workspace NULL, misaligned or smaller than psk_workspace_bytes */
    PSK_ERR_UNSUPPORTED = 5, /* unknown op / variant / phases */
    PSK_ERR_HIP = 6,         /* the HIP runtime reported an error at launch */
    PSK_ERR_ALIGNMENT = 7    /* BCSR: vals (and x for SpMV) not 16-byte aligned; fp64 SpMV: an operand not 8-byte aligned */
} psk_status;

typedef enum {
    PSK_OP_SPMV_CSR = 0,
    PSK_OP_SPMM_CSR = 1,
    PSK_OP_SPMV_BCSR = 2,
    PSK_OP_SPMM_BCSR = 3,
    PSK_OP_MTTKRP_CSF3 = 4,
    PSK_OP_SPMV_CSR_F64 = 5
} psk_op;

enum { PSK_PHASE_PARTITION = 1, PSK_PHASE_MAIN = 2, PSK_PHASE_FIXUP = 4, PSK_PHASE_ALL = 7 };

/* How psk_partition_csr locates the tile starts (Section 5, "Divide": an O(log n) search per tile or an
 * O(n) walk).  Both give the same table. */
enum { PSK_PARTITION_AUTO = 0, PSK_PARTITION_SEARCH = 1, PSK_PARTITION_SCAN = 2 };

/* Row-split (coordinate-space) baselines, Section 8.3 and the appendix schedules
 * "SpMV Thread per Row on GPU" / "SpMV Warp per Row on GPU". */
enum { PSK_ROWSPLIT_THREAD_PER_ROW = 0, PSK_ROWSPLIT_WAVE_PER_ROW = 1 };

const char *psk_status_string(int status);

/* Library version as major*10000 + minor*100 + patch. */
int psk_version(void);

/* Default position-tile size of an operation (what tile = 0 selects); -1 for an unknown op.
 * For the BCSR operations the unit is blocks. */
int32_t psk_default_tile(int op);
/* The same for a BCSR operation with block edge bs (the SpMV tile sets differ with bs); -1 if unsupported. */
int32_t psk_default_tile_bcsr(int op, int32_t bs);

/* ceil(nnz / tile): number of tiles of the position cut; 0 when nnz <= 0; -1 when tile <= 0. */
int64_t psk_num_tiles(int64_t nnz, int32_t tile);

/*
 * Bytes of workspace an operation needs (tile-row table, one carry record per
 * tile, a second table for the two-level cut, one column range per tile and wave).  `k` is the number of dense columns (ignored for SpMV), `bs` the BCSR
 * block edge (ignored for CSR), `tile` as passed to the operation (0 = default).
 * Returns 0 on invalid arguments.  Always at least 256.
 */
size_t psk_workspace_bytes(int op, int64_t rows, int64_t nnz, int32_t k, int32_t bs, int32_t tile);

/*
 * The position cut (Section 3 "tiling the position space"; Section 5 "Split";
 * Section 6.2: the first coordinate of a tile is found by binary search).
 *   tile_row[t] = max { i in [0, rows] : pos[i] <= min(t*tile, nnz) },  t = 0 .. ntiles
 * i.e. for t < ntiles the (non-empty) row that owns the tile's first position, and
 * tile_row[ntiles] = rows.  tile_row has psk_num_tiles(nnz, tile) + 1 int32 entries.
 * Any tile >= 1 is accepted here.  nnz = 0 gives the single entry [rows].
 * method: PSK_PARTITION_SEARCH runs one binary search over pos per table entry;
 * PSK_PARTITION_SCAN reads pos once and lets every non-empty row write the entries of the tile
 * starts it contains (no dependent loads; faster unless pos is very large and the tiles are few);
 * PSK_PARTITION_AUTO picks one from rows and the number of tiles.  The operations below use AUTO.
 */
int psk_partition_csr(int64_t rows, int64_t nnz, const int32_t *pos, int32_t tile, int method,
                      int32_t *tile_row, void *stream);

/*
 * y = A x, CSR, position-space schedule (appendix "SPMV on a GPU"): one workgroup
 * per tile of `tile` positions; coalesced loads of crd/vals, gather of x, products
 * kept in registers (the schedule's precompute + unroll), reduction per row inside
 * the tile, one carry record per tile for a row that began in an earlier tile
 * (instead of the schedule's atomics), carries added by a second small kernel.
 * x has cols entries, y rows entries.  tile in {0, 256, 512, 1024, 2048, 4096}; 0 means 2048, or
 * 1024 when col_passes > 1 (psk_workspace_bytes with tile = 0 covers both).  With tile = 0, col_passes <= 1
 * and nnz <= 16384 the whole matrix is taken as one tile by one workgroup: one launch (in PSK_PHASE_MAIN),
 * no table, no carries; such problems are bound by launch latency.
 *
 * col_passes (0 or 1 = off, at most PSK_MAX_COL_PASSES): the main step is run that many times, pass q
 * gathering only the columns of the q-th equal slice of [0, cols) and adding to what the earlier passes
 * stored (the first pass records each tile's column range, and a later pass leaves a tile whose range
 * misses its window untouched).  A and the row bounds are streamed once per pass; in exchange the slice
 * of x a pass gathers from can stay in the 4 MB L2 of a die.  Worth it only for matrices whose columns are scattered over
 * an x larger than that (a gather that misses L2 moves a 128-byte line for 4 useful bytes); it is a
 * loss for banded or otherwise local matrices.  psk_analyze_csr suggests a value.  Results stay
 * deterministic; they differ from the single-pass result within the usual fp32 reassociation.
 */
int psk_spmv_csr(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd,
                 const float *vals, const float *x, float *y, int32_t tile, int32_t col_passes, int phases,
                 void *workspace, size_t workspace_bytes, void *stream);

/*
 * psk_spmv_csr for callers that cannot allocate device memory and have no workspace to pass: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same product (all three phases), same
 * kernels and bit-identical results as psk_spmv_csr with the same tile and col_passes; the table, the carry
 * records, the column ranges and the run list live in a built-in device array of PSK_STATIC_SCRATCH_BYTES (4 MiB per GPU,
 * held until the process ends) instead of a caller's workspace.  The call allocates nothing.
 *  - Limit: psk_workspace_bytes(PSK_OP_SPMV_CSR, rows, nnz, 1, 1, tile) must not exceed
 *    psk_static_scratch_bytes(), i.e. about 74 000 tiles (153 M nonzeros at tile 2048, 76 M at 1024);
 *    beyond that PSK_ERR_WORKSPACE and nothing is enqueued.
 *  - tile in {0, 256, 512, 1024, 2048, 4096}; 0 means 2048, or 1024 when col_passes > 1.
 *  - All calls on one GPU share that GPU's array: calls that may overlap in time on one GPU (different
 *    streams, or different host threads without stream ordering) race on it; order them on one stream.
 *    The array keeps the last call's contents; a product overwrites every entry it later reads.
 *  - The device used is the current device of the calling thread; `stream` must belong to it.
 */
#define PSK_STATIC_SCRATCH_BYTES (4u << 20)
size_t psk_static_scratch_bytes(void);
int psk_spmv_csr_static(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd,
                        const float *vals, const float *x, float *y, int32_t tile, int32_t col_passes,
                        void *stream);

/*
 * Suggests col_passes for psk_spmv_csr on this matrix (like the tile->row table it depends only on A and
 * can be kept).  Answers 1 when x fits a die's L2 or the matrix is small; otherwise it samples up to
 * 16384 positions and, if fewer than half of them have their successor's column in the same 128-byte
 * line of x, suggests ceil(4*cols bytes / 6 MiB), at most PSK_MAX_COL_PASSES.
 * A suggestion above 1 also marks the matrices for which the column-slab copy (psk_slab_build_csr, then
 * psk_spmv_slab) pays once the matrix is multiplied about ten times or more.
 * `col_passes` is a HOST pointer.  This call SYNCHRONISES `stream` when it samples (it reads the count
 * back); `workspace` needs 256 bytes.
 */
#define PSK_MAX_COL_PASSES 4
int psk_analyze_csr(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd,
                    void *workspace, size_t workspace_bytes, int32_t *col_passes, void *stream);

/*
 * Checks the preconditions the operations do not check (they would read or write out of bounds on a
 * malformed structure).  *violation (HOST pointer) receives 0 if pos[0] = 0, pos is non-decreasing,
 * pos[rows] = nnz and 0 <= crd[p] < cols for all p; otherwise the number of the first condition, in that
 * order, that fails: 1, 2, 3 or 4.  Works for BCSR (pass block counts) and for each level of the
 * compressed tensor formats.  One pass over pos and crd; SYNCHRONISES `stream` (it reads the counts
 * back); `workspace` needs 256 bytes.  Note that the kernel itself trusts nnz and rows as array lengths.
 */
int psk_validate_csr(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd,
                     void *workspace, size_t workspace_bytes, int32_t *violation, void *stream);

/*
 * Which schedule for y = A x on this matrix: the position cut (psk_spmv_csr) or the row split with one
 * wave per row (psk_spmv_csr_rowsplit)?  Section 8.4 shows that the answer depends on the skew of the
 * row lengths.  Rule, from sweeps on MI355X: the row split only when the matrix is small
 * (nnz <= 6 * 2^20, where the position path's partition and fix-up launches are a visible share), the
 * mean row has at least 48 entries (a wave is mostly busy) and the longest row is at most 3.5 times the
 * mean; otherwise the position cut.  `schedule` is a HOST pointer and receives PSK_SCHEDULE_*.
 * Like psk_analyze_csr this call SYNCHRONISES `stream` when it has to look at pos (it reads the longest
 * row back); `workspace` needs 256 bytes.
 */
enum { PSK_SCHEDULE_POSITIONS = 0, PSK_SCHEDULE_ROWS = 1 };
int psk_suggest_schedule_csr(int64_t rows, int64_t nnz, const int32_t *pos, void *workspace,
                             size_t workspace_bytes, int32_t *schedule, void *stream);

/*
 * C = A B, CSR A, position-space schedule (appendix "SPMM on a GPU"): positions are
 * split over workgroups and waves, the columns of B over the lanes of a wave, the
 * loop over a wave's positions is innermost.  B is cols x k with row stride ldb
 * (>= k), C is rows x k with row stride ldc (>= k), both in floats.  Any k >= 1
 * (k <= 32 runs a variant in which 2, 4 or 8 groups of lanes take consecutive positions).
 * tile in {0, 256, 512, 1024, 2048}.
 */
int psk_spmm_csr(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd,
                 const float *vals, const float *B, int32_t k, int64_t ldb, float *C, int64_t ldc,
                 int32_t tile, int phases, void *workspace, size_t workspace_bytes, void *stream);

/*
 * BCSR (Section 1): brows x bcols blocks of bs x bs floats, nblocks stored blocks;
 * pos/crd index blocks; the position cut is taken at the block level (Section 3:
 * a cut may be placed at any level of the hierarchy), `tile` counts blocks.
 * x has bcols*bs entries, y brows*bs.  bs in {2, 4, 8} (other sizes: PSK_ERR_UNSUPPORTED).
 * vals must be 16-byte aligned, x 16-byte (bs = 2: 8-byte) aligned.
 * tile (0 = default): bs = 4: {64, 128, 256, 512}, default 512; bs = 2: {512, 1024, 2048}, default 1024;
 * bs = 8: {32, 64, 128}, default 64.  Workspace: psk_workspace_bytes(PSK_OP_SPMV_BCSR, brows, nblocks, 1, bs, tile).
 */
int psk_spmv_bcsr(int64_t brows, int64_t bcols, int64_t nblocks, int32_t bs, const int32_t *pos,
                  const int32_t *crd, const float *vals, const float *x, float *y, int32_t tile,
                  int phases, void *workspace, size_t workspace_bytes, void *stream);

/* C = A B with BCSR A: B is (bcols*bs) x k, C is (brows*bs) x k.  bs in {2, 4, 8}.
 * vals must be 16-byte aligned.  tile in {0, 64, 128, 256, 512}. */
int psk_spmm_bcsr(int64_t brows, int64_t bcols, int64_t nblocks, int32_t bs, const int32_t *pos,
                  const int32_t *crd, const float *vals, const float *B, int32_t k, int64_t ldb,
                  float *C, int64_t ldc, int32_t tile, int phases, void *workspace,
                  size_t workspace_bytes, void *stream);

/*
 * MTTKRP, A(i,j) = B(i,k,l) * C(k,j) * D(l,j)  (appendix "MTTKRP on a GPU"), B an order-3 tensor stored as a
 * three-level coordinate hierarchy (Section 3), one level per mode:
 *   slices  s = 0 .. nslices-1 (mode i): coordinate crd_i[s], or s itself when crd_i is NULL (dense first
 *           level; then nslices must equal dim_i); slice s owns fibers pos_k[s] .. pos_k[s+1];
 *   fibers  q = 0 .. nfibers-1 (mode k): coordinate crd_k[q]; fiber q owns leaves pos_l[q] .. pos_l[q+1];
 *   leaves  p = 0 .. nnz-1     (mode l): coordinate crd_l[p], value vals[p].
 * Preconditions like CSR at each level: pos_k[0] = 0, pos_k[nslices] = nfibers, pos_l[0] = 0,
 * pos_l[nfibers] = nnz, both non-decreasing, coordinates in range; crd_i (if given) distinct.  Empty slices
 * and empty fibers are allowed.
 * C is dim_k x j (row stride ldc), D is dim_l x j (ldd), A is dim_i x j (lda), all row-major fp32.  Every
 * row of A is assigned (rows without leaves become 0).  Schedule: fuse (k,l), fuse with i, cut the fused loop
 * in the position space of the LEAF level into tiles of `tile` leaves, j over the lanes of a wave; the two
 * levels above the cut are tracked per tile (psk_partition_csf3) and inside the tile.
 * tile in {0, 256, 512, 1024, 2048}; workspace from psk_workspace_bytes(PSK_OP_MTTKRP_CSF3, nslices, nnz, j, 1, tile).
 */
int psk_mttkrp_csf3(int64_t dim_i, int64_t dim_k, int64_t dim_l, int64_t nslices, int64_t nfibers, int64_t nnz,
                    const int32_t *crd_i, const int32_t *pos_k, const int32_t *crd_k, const int32_t *pos_l,
                    const int32_t *crd_l, const float *vals, const float *C, int64_t ldc, const float *D,
                    int64_t ldd, int32_t j, float *A, int64_t lda, int32_t tile, int phases, void *workspace,
                    size_t workspace_bytes, void *stream);

/*
 * The position cut of the leaf level of that hierarchy.  For t = 0 .. ntiles (ntiles = ceil(nnz / tile)):
 *   tile_fiber[t] = max { q in [0, nfibers] : pos_l[q] <= min(t*tile, nnz) }
 *   tile_slice[t] = max { s in [0, nslices] : pos_k[s] <= tile_fiber[t] }
 * i.e. the fiber and the slice that own the tile's first leaf (two chained binary searches, Section 6.2),
 * with the sentinels (nfibers, nslices) in the last entry.  Both tables have ntiles + 1 int32 entries.
 */
int psk_partition_csf3(int64_t nslices, int64_t nfibers, int64_t nnz, const int32_t *pos_k, const int32_t *pos_l,
                       int32_t tile, int32_t *tile_slice, int32_t *tile_fiber, void *stream);

/*
 * Coordinate-space baselines (Section 3 "tiling the coordinate space"; Section 8.3):
 * rows are split over workgroups, no search, unequal work per tile.  No workspace.
 * variant = PSK_ROWSPLIT_THREAD_PER_ROW or PSK_ROWSPLIT_WAVE_PER_ROW.
 */
int psk_spmv_csr_rowsplit(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos,
                          const int32_t *crd, const float *vals, const float *x, float *y,
                          int variant, void *stream);

/*
 * y = A x with fp64 values, vector and result (the value type of the paper's own schedules: the
 * per-thread temporary of appendix "SPMV on a GPU" is Float64).  Same cut, tile kernel structure,
 * carry records (doubles) and fix-up as psk_spmv_csr, column passes included (col_passes as there; x is
 * twice as large per column, so slices of the same byte size hold half the columns); products and sums in fp64.
 * vals [nnz], x [cols], y [rows] doubles, 8-byte aligned (PSK_ERR_ALIGNMENT otherwise); crd and vals
 * 16-byte aligned selects the 16-byte load path.  tile in {0, 256, 512, 1024, 2048}, 0 = 1024.
 * Workspace from psk_workspace_bytes(PSK_OP_SPMV_CSR_F64, rows, nnz, 1, 1, tile).
 * Deterministic; |y - exact| <= 1e-14 * sum_j |a_ij x_j| per row.
 */
int psk_spmv_csr_f64(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd,
                     const double *vals, const double *x, double *y, int32_t tile, int32_t col_passes,
                     int phases, void *workspace, size_t workspace_bytes, void *stream);

/*
 * y = A x with A in DCSR, the doubly compressed form for hypersparse matrices (Section 2 names it next
 * to CSR; Section 3, last paragraphs: a position cut can be taken at any level of the hierarchy).
 * Only `nstored` rows are stored: crd_i [nstored] holds their coordinates (strictly increasing, in
 * [0, rows)), pos [nstored + 1], crd and vals [nnz] are as in CSR but indexed by stored row.  y has
 * `rows` entries; rows that are not stored (and stored rows without entries) become +0.
 *   cut = PSK_CUT_POSITIONS: tiles of `tile` positions of the column level (equal work per tile; a row
 *         may be divided; table, carries and fix-up as in psk_spmv_csr, the table holds stored-row
 *         indices).  tile, col_passes, workspace: as psk_spmv_csr with rows = nstored (psk_analyze_csr
 *         with rows = nstored suggests col_passes).
 *   cut = PSK_CUT_ROWS: tiles of four positions of the row level, one wave per stored row (equal
 *         number of stored rows per tile; no row is divided, so no table, no carries, no fix-up:
 *         only PSK_PHASE_MAIN does anything).  `tile` must still be a valid value (0 is); col_passes is
 *         ignored.
 * The main phase zero-fills y first.
 */
enum { PSK_CUT_POSITIONS = 0, PSK_CUT_ROWS = 1 };
int psk_spmv_dcsr(int64_t rows, int64_t cols, int64_t nstored, int64_t nnz, const int32_t *crd_i,
                  const int32_t *pos, const int32_t *crd, const float *vals, const float *x, float *y,
                  int cut, int32_t tile, int32_t col_passes, int phases, void *workspace, size_t workspace_bytes,
                  void *stream);

/*
 * y = A x, CSR, with the position space DIVIDED instead of split (Section 5 "Divide": the number of
 * pieces is fixed, so the number of searches for a piece's first coordinate does not grow with the
 * matrix).  `parts` persistent workgroups (0 = 2048; fewer when the matrix has fewer than that many
 * chunks of 2048 positions), each of which finds its first row with one binary search inside the
 * kernel, then walks its equal share of the positions chunk by chunk and tracks the rows (Section 6.2).
 * No table and no partition step (PSK_PHASE_PARTITION does nothing); one carry record per part, added
 * by the same fix-up as psk_spmv_csr.  Workspace: psk_workspace_bytes(PSK_OP_SPMV_CSR, rows, nnz, 1, 1,
 * 2048) or more.  Same result bar as psk_spmv_csr; deterministic for a given `parts`.
 */
int psk_spmv_csr_divide(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd,
                        const float *vals, const float *x, float *y, int32_t parts, int phases,
                        void *workspace, size_t workspace_bytes, void *stream);

/*
 * Baseline with the schedule's own race strategy (appendix "SPMV on a GPU": the thread level is
 * parallelised with OutputRaceStrategy::Atomics; Section 6.3, first strategy): same position cut and tile
 * kernel as psk_spmv_csr, but y is zero-filled first and the part of a row that other tiles also hold is
 * added with a floating-point atomic instead of going through a carry record.  No fix-up step
 * (PSK_PHASE_FIXUP is ignored).  The order of the atomic adds is not fixed, so rows that span tiles are
 * NOT bit-reproducible from run to run; they stay within the fp32 tolerance.  Same workspace as
 * psk_spmv_csr (only the tile->row table is used).
 */
int psk_spmv_csr_atomics(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd,
                         const float *vals, const float *x, float *y, int32_t tile, int phases,
                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * Ablation of Section 8.3 (the optimised schedule "without the temporary or loop unrolling"): same cut,
 * same row logic, carries and fix-up as psk_spmv_csr, but each thread walks its positions in a rolled
 * loop (load, gather, multiply, store to on-chip memory, one position after the other) instead of
 * issuing all its loads first and keeping the products in registers.  Same arguments, workspace and
 * result (within the fp32 tolerance) as psk_spmv_csr with col_passes = 1.
 */
int psk_spmv_csr_notemp(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd,
                        const float *vals, const float *x, float *y, int32_t tile, int phases,
                        void *workspace, size_t workspace_bytes, void *stream);

/* Row-split SpMM baseline: one wave per row, lanes over the columns of B. */
int psk_spmm_csr_rowsplit(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos,
                          const int32_t *crd, const float *vals, const float *B, int32_t k,
                          int64_t ldb, float *C, int64_t ldc, void *stream);

/*
 * ---- y = A x over a column-slab copy of A (an analysis step, then products) ----
 *
 * Section 8.6 of the paper obtains locality by tiling: split a loop and move its outer part outward;
 * Section 3 lets the position cut be taken in any coordinate hierarchy.  Here the column loop j is split
 * by slabs of PSK_SLAB_COLS columns, jo = j / PSK_SLAB_COLS moves outermost and A is stored once in that
 * order: three levels (jo dense, i compressed, ji compressed) whose leaf positions ("slots") are the CSR
 * positions bucketed stably by slab.  The leaf position space is divided into equal pieces as in
 * psk_spmv_csr_divide, but a piece needs one slab of x only, which a workgroup keeps in on-chip memory, so
 * the gathers of x never leave the compute unit.  Meant for matrices whose columns are scattered over an x
 * that exceeds the caches (where a gather costs a cache-line request per entry); for banded matrices
 * psk_spmv_csr is the better choice.
 *
 * Structure (psk_slab; the arrays live in the caller's `mem`, the struct itself is host memory):
 *   - every slab is padded with empty slots (value 0, column 0) to a multiple of PSK_SLAB_CHUNK slots;
 *     nslots = all slots, nchunks = nslots / PSK_SLAB_CHUNK; slab_chunk[s] = first chunk of slab s
 *     (nslabs + 1 entries);
 *   - a pair is a maximal run of slots of one row inside one chunk; scol[j] holds slot j's column inside the
 *     slab (low 15 bits), bit 15 is set on the last slot of a pair; the slot's value is svals[v(j)], where
 *     v permutes the slots inside each chunk (slot 8l + k of a chunk sits at (k / 4) * 256 + 4l + k % 4 of the
 *     chunk, so that 64 lanes that own 8 consecutive slots each fetch them with two contiguous loads; with
 *     8-byte values at (k / 2) * 128 + 2l + k % 2: four loads);
 *     chunk_pair[c] = index of the pair of chunk c's first slot (nchunks + 1 entries, last = npairs);
 *   - qpos[rows + 1], qidx[nq]: the pairs of each row, in the order of their first slots in the CSR;
 *     qtile_row: the position cut (psk_partition_csr) of (qpos, nq) with tiles of `tile` pairs.
 * Product: step 1 writes P[pair] = sum of value * x over the pair's slots; step 2 is y = (qpos, qidx) * P
 * with unit values through the tile kernel, carries and fix-up of psk_spmv_csr.  Deterministic; same
 * result bar as psk_spmv_csr.  Columns inside a row need not be sorted or distinct.
 *
 * Limits: cols <= 8192 * PSK_SLAB_COLS, nnz + 511 * nslabs < 2^31, nslabs * ceil(nnz / 2048) <= 2^30
 * (PSK_ERR_UNSUPPORTED / PSK_ERR_SIZE otherwise).
 *
 * fp64 values (the value type of the paper's own schedules, appendix "SPMV on a GPU"): the _f64 entry points
 * build and use the same structure with 8-byte values and slabs of PSK_SLAB_COLS_F64 columns (a slab of x and
 * the staging area of the pair sums share the 160 KB of on-chip memory); x, y and the pair sums are doubles.
 */
#define PSK_SLAB_COLS 32736
#define PSK_SLAB_COLS_F64 16352
#define PSK_SLAB_CHUNK 512
typedef struct psk_slab {
    int64_t rows, cols, nnz;
    int64_t nslabs, nslots, nchunks, npairs, nq;
    int32_t slab_cols, chunk, tile, value_bytes;   /* value_bytes: 4 (float) or 8 (double) */
    const void *svals;           /* [nslots] floats or doubles, device */
    const uint16_t *scol;        /* [nslots]  device */
    const int32_t *chunk_pair;   /* [nchunks + 1] device */
    const int32_t *slab_chunk;   /* [nslabs + 1]  device */
    const int32_t *qpos;         /* [rows + 1]    device */
    const int32_t *qidx;         /* [nq]          device */
    const int32_t *qtile_row;    /* [ceil(nq / tile) + 1] device */
} psk_slab;

/* Bytes of device memory for the structure of a rows x cols matrix with nnz entries (an upper bound: the
 * exact size depends on how the entries fall into slabs and chunks; about 10 bytes per entry + 4 per row; with fp64 values about 14 per entry);
 * 0 when the sizes are outside the limits above. */
size_t psk_slab_mem_bytes(int64_t rows, int64_t cols, int64_t nnz);
size_t psk_slab_mem_bytes_f64(int64_t rows, int64_t cols, int64_t nnz);
/* Bytes of scratch memory psk_slab_build_csr needs (about 16 bytes per entry); free to reuse afterwards. */
size_t psk_slab_build_workspace_bytes(int64_t rows, int64_t cols, int64_t nnz);
size_t psk_slab_build_workspace_bytes_f64(int64_t rows, int64_t cols, int64_t nnz);
/* Bytes of workspace a product over S needs (the pair sums and the carry records); 0 if S is NULL. */
size_t psk_slab_spmv_workspace_bytes(const psk_slab *S);

/*
 * The analysis step: builds the structure from a CSR matrix, entirely on the device (a histogram of the
 * slabs per block of 2048 positions, prefix sums, a stable scatter, the pairs of every chunk and their prefix sums, the
 * row lists and their position cut).  `mem` (psk_slab_mem_bytes, 256-byte aligned) receives the arrays and
 * must stay allocated while *out is used; `workspace` (psk_slab_build_workspace_bytes, 256-byte aligned) is
 * scratch.  *out (HOST pointer) receives the sizes and the device pointers.  pos, crd, vals: as for
 * psk_spmv_csr (same unchecked preconditions).  This call SYNCHRONISES `stream` (it reads three counts
 * back).  The structure depends only on A: build once, multiply many times.
 */
int psk_slab_build_csr(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd,
                       const float *vals, void *mem, size_t mem_bytes, void *workspace, size_t workspace_bytes,
                       psk_slab *out, void *stream);
/* The same for fp64 values (8-byte aligned, PSK_ERR_ALIGNMENT otherwise); sizes from the _f64 size functions. */
int psk_slab_build_csr_f64(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd,
                           const double *vals, void *mem, size_t mem_bytes, void *workspace,
                           size_t workspace_bytes, psk_slab *out, void *stream);

/*
 * y = A x over the structure: x has S->cols entries, y S->rows entries (assigned, rows without entries
 * become +0).  `workspace`: psk_slab_spmv_workspace_bytes(S), 256-byte aligned; products that may overlap in
 * time need separate workspaces, the structure itself is only read.  Enqueues three kernels on `stream`
 * (pair sums, row sums, carry fix-up) and returns; allocates nothing, never synchronises.  `phases`:
 * PSK_PHASE_MAIN = the two sum kernels, PSK_PHASE_FIXUP = the fix-up (PSK_PHASE_ALL for a product;
 * PSK_PHASE_PARTITION does nothing: the cut of the row lists is part of the structure).
 * PSK_ERR_SIZE for a struct whose sizes are not consistent with each other (they decide grids and index ranges);
 * what the arrays hold is the caller's contract: only psk_slab_build_csr makes them.
 */
int psk_spmv_slab(const psk_slab *S, const float *x, float *y, int phases, void *workspace,
                  size_t workspace_bytes, void *stream);
/* The same over a structure built by psk_slab_build_csr_f64 (PSK_ERR_SIZE for a structure of the other value
 * type); x and y doubles, 8-byte aligned; products and sums in fp64; result bar as psk_spmv_csr_f64. */
int psk_spmv_slab_f64(const psk_slab *S, const double *x, double *y, int phases, void *workspace,
                      size_t workspace_bytes, void *stream);

/*
 * ---- per-CU load balance (instrumented build only) ----
 *
 * The library can be built a second time with -DPSK_CU_TRACE (libpsk_trace.so, python -m paper_2001_00532_amd.build
 * makes both).  In that build every workgroup of the CSR SpMV tile kernel, of the two row-split kernels and of the
 * slab pair kernel writes a record of three 64-bit words: its start and its end on the 100 MHz wall clock, and
 * (HW_ID & 0xffff) | (XCC_ID << 32), i.e. the compute unit it ran on.  Workgroup b of the slab pair kernel writes
 * record b (b < PSK_CU_TRACE_SLAB_RECORDS), workgroup b of the other kernels record PSK_CU_TRACE_SLAB_RECORDS + b, so
 * that a product over the slab structure, which launches both kinds, can be traced in one go.  The host forms the busy
 * time of each compute unit from them (Section 3 of the paper: equal position tiles give static load balance; the
 * trace shows it per CU, position cut against row split).  records = NULL switches tracing off.  The records must be
 * zeroed by the caller before each traced launch (the end time is written with an atomic max); workgroups beyond
 * nrecords are not recorded.  Synchronous (it copies the pointer to the device).  The tracing costs time: use
 * ratios, not absolute times.  The plain build returns PSK_ERR_UNSUPPORTED.
 */
#define PSK_CU_TRACE_SLAB_RECORDS 1024
int psk_cu_trace_set(void *records, size_t nrecords);

/*
 * ---- calibration kernels (no product; they reproduce the machine rates the design is argued with) ----
 *
 * psk_calibrate_stream_read: reads `bytes` bytes at `src` (16-byte aligned) once with 16-byte non-temporal
 *   loads; nothing is written (`sink` needs one float).  Rate = bytes / kernel time: the practical ceiling
 *   of a read-only stream.
 * psk_calibrate_gather: out[i/8] (n/8 floats) receives sums of table[idx[i]], n gathers of 4-byte words
 *   with 16-byte loads of the int32 indices (0 <= idx < table_elems, caller's contract), 2048 gathers per
 *   workgroup: the CSR tile kernel's access pattern without values and row logic.  n must be a positive
 *   multiple of 2048, idx 16-byte aligned.  Time / n = cost of one gather for that table size.
 * psk_calibrate_gather_lds: the same number of gathers from a table of at most PSK_SLAB_COLS floats that
 *   every workgroup first copies into on-chip memory; 16-bit indices (idx < table_elems), n a positive
 *   multiple of 8192, out has 1024 floats per workgroup (at most 256 workgroups).
 * All three only enqueue one kernel on `stream`.
 */
int psk_calibrate_stream_read(const void *src, size_t bytes, float *sink, void *stream);
int psk_calibrate_gather(const float *table, int64_t table_elems, const int32_t *idx, int64_t n, float *out,
                         void *stream);
int psk_calibrate_gather_lds(const float *table, int32_t table_elems, const uint16_t *idx, int64_t n, float *out,
                             void *stream);

#ifdef __cplusplus
}
#endif
#endif /* PSK_H */
