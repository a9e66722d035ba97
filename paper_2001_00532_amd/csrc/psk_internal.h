// Host-side declarations shared between the C-ABI layer (api.hip) and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include <tuple>
#include <utility>

namespace psk {

// Kernel launches go through hipLaunchKernel so that each launcher reports the status of ITS launches only:
// the global "last error" of the runtime may hold (and reading it would clear) an error left by the caller's
// own earlier HIP calls.  A launcher may launch several kernels; the first failure is kept per host thread
// and handed out (and reset) by take_launch_status().
extern thread_local hipError_t tls_launch_status;
inline hipError_t take_launch_status()
{
    const hipError_t e = tls_launch_status;
    tls_launch_status = hipSuccess;
    return e;
}
template <typename... KA, size_t... I>
inline hipError_t launch_tuple(void (*kern)(KA...), dim3 grid, dim3 block, unsigned shmem, hipStream_t s,
                               std::tuple<KA...> &args, std::index_sequence<I...>)
{
    void *ptrs[sizeof...(KA) ? sizeof...(KA) : 1] = {static_cast<void *>(&std::get<I>(args))...};
    return hipLaunchKernel(reinterpret_cast<const void *>(kern), grid, block, ptrs, shmem, s);
}
template <typename... KA, typename... A>
inline void launch_kernel(void (*kern)(KA...), dim3 grid, dim3 block, unsigned shmem, hipStream_t s, A &&...a)
{
    static_assert(sizeof...(KA) == sizeof...(A), "argument count does not match the kernel's parameters");
    std::tuple<KA...> args{static_cast<KA>(a)...};
    const hipError_t e = launch_tuple(kern, grid, block, shmem, s, args, std::index_sequence_for<KA...>{});
    if (e != hipSuccess && tls_launch_status == hipSuccess) tls_launch_status = e;
}
#define PSK_LAUNCH(kern, grid, block, shmem, stream, ...) \
    ::psk::launch_kernel(kern, grid, block, shmem, stream, __VA_ARGS__)

// Workspace carving: [tile_row: ntiles+1 int32][carry_row: ntiles int32][carry_val: ntiles*width float]
// [tile_aux: ntiles+1 int32 (second table of a two-level cut)][tile_cols: ntiles*8 int32 (column range of each
// tile, one min/max pair per wave, written by the first column pass)][gap: 2+2*ntiles int32 (the long runs of
// empty rows that the fix-up step clears with many workgroups)], each part starting on a 256-byte boundary.
struct Workspace {
    int32_t *tile_row;
    int32_t *carry_row;
    float   *carry_val;
    int32_t *tile_aux;
    int32_t *tile_cols;
    int32_t *gap;        // [2 + 2*ntiles]: count, arrivals, then (first row, end row) of every long run of rows a tile spans
    size_t   bytes;
};
inline size_t align256(size_t n) { return (n + 255) & ~size_t(255); }
inline Workspace carve(void *base, int64_t ntiles, int64_t width)
{
    Workspace w;
    char *p = static_cast<char *>(base);
    size_t a = align256(size_t(ntiles + 1) * 4), b = align256(size_t(ntiles) * 4 + 4),
           c = align256(size_t(ntiles) * size_t(width) * 4 + 4);
    w.tile_row = reinterpret_cast<int32_t *>(p);
    w.carry_row = reinterpret_cast<int32_t *>(p + a);
    w.carry_val = reinterpret_cast<float *>(p + a + b);
    const size_t d = align256(size_t(ntiles) * 32 + 4);
    w.tile_aux = reinterpret_cast<int32_t *>(p + a + b + c);
    w.tile_cols = reinterpret_cast<int32_t *>(p + a + b + c + a);
    const size_t g = align256(size_t(ntiles) * 8 + 8);
    w.gap = reinterpret_cast<int32_t *>(p + a + b + c + a + d);
    w.bytes = a + b + c + a + d + g;
    return w;
}

// Every launcher enqueues on `s` and returns the status of its own launches (take_launch_status()).

// gap (optional): the run list of the workspace; its two counters are cleared here
hipError_t launch_partition(int64_t rows, int64_t nnz, const int32_t *pos, int32_t tile, int method,
                            int32_t *tile_row, hipStream_t s, int32_t *gap = nullptr);
hipError_t launch_fill_zero(float *p, int64_t n, hipStream_t s);
hipError_t launch_fill_zero_2d(float *p, int64_t rows, int32_t width, int64_t ld, hipStream_t s);
hipError_t launch_validate_csr(int32_t rows, int32_t cols, int32_t nnz, const int32_t *pos, const int32_t *crd,
                               int32_t *result, hipStream_t s);
hipError_t launch_max_row(int32_t rows, const int32_t *pos, int32_t *result, hipStream_t s);
hipError_t launch_probe_locality(int32_t nnz, const int32_t *crd, int32_t *result, hipStream_t s);
// Adds the per-tile carry records to the output: element e of a record of `nsub*k` floats goes to
// out[(row*nsub + e / k) * ld + e % k].
// `pos2` (optional): two-level hierarchy, a row's last position is pos2[pos[r+1]] - 1.  `rowmap` (optional):
// row r of the hierarchy is stored at output row rowmap[r].
// gaps = true (CSR SpMV only): extra workgroups clear the long runs of empty rows that the tile kernel listed in w.gap
hipError_t launch_carry_fixup(int32_t ntiles, int32_t nsub, int32_t k, int64_t ld, int32_t tile, const int32_t *pos,
                              const Workspace &w, float *out, hipStream_t s, const int32_t *pos2 = nullptr,
                              const int32_t *rowmap = nullptr, bool gaps = false);
// A tile whose rows span more than this many rows does not walk them: it finds the rows of its positions by search
// and leaves the run of empty rows to the fix-up step (which clears it with many workgroups).
constexpr int32_t kGapRows = 32768;
constexpr int32_t kGapFillGroups = 512;

// CSR SpMV
bool spmv_csr_tile_ok(int32_t tile);
hipError_t launch_spmv_csr_main(int32_t rows, int32_t cols, int32_t nnz, const int32_t *pos, const int32_t *crd,
                                const float *vals, const float *x, float *y, int32_t tile, int32_t col_passes,
                                const Workspace &w, hipStream_t s, const int32_t *rowmap = nullptr, bool gaps = false);
// the whole matrix as one tile of one workgroup (nnz <= kSingleTile): no table, no carries
constexpr int32_t kSingleTile = 16384;
hipError_t launch_spmv_csr_single(int32_t rows, int32_t cols, int32_t nnz, const int32_t *pos, const int32_t *crd,
                                  const float *vals, const float *x, float *y, hipStream_t s);
// rowmap (optional, both launchers): row r of the hierarchy is row rowmap[r] of y (DCSR)
hipError_t launch_spmv_rowsplit(int32_t rows, const int32_t *pos, const int32_t *crd, const float *vals,
                                const float *x, float *y, int variant, hipStream_t s,
                                const int32_t *rowmap = nullptr);

// CSR SpMV with the position space divided into `parts` pieces of chunks_per_part * 2048 positions
// (persistent workgroups, in-kernel search, no table); carry records: one per part
constexpr int32_t kDivideChunk = 2048;
hipError_t launch_spmv_csr_divide(int32_t rows, int32_t cols, int32_t nnz, const int32_t *pos, const int32_t *crd,
                                  const float *vals, const float *x, float *y, int32_t parts,
                                  int32_t chunks_per_part, const Workspace &w, hipStream_t s);

// CSR SpMV, fp64 operands (carry records are doubles: the workspace is carved with width 2)
bool spmv_csr_f64_tile_ok(int32_t tile);
hipError_t launch_spmv_csr_f64_main(int32_t rows, int32_t cols, int32_t nnz, const int32_t *pos, const int32_t *crd,
                                    const double *vals, const double *x, double *y, int32_t tile, int32_t col_passes,
                                    const Workspace &w, hipStream_t s, bool gaps = false);
hipError_t launch_carry_fixup_f64(int32_t ntiles, int32_t tile, const int32_t *pos, const Workspace &w, double *out,
                                  hipStream_t s, bool gaps = false);

// CSR SpMM
bool spmm_csr_tile_ok(int32_t tile);
hipError_t launch_spmm_csr_main(int32_t rows, int32_t nnz, const int32_t *pos, const int32_t *crd,
                                const float *vals, const float *B, int32_t k, int64_t ldb, float *C,
                                int64_t ldc, int32_t tile, const Workspace &w, hipStream_t s);
// k <= 32: the wave is split into groups that take consecutive positions
hipError_t launch_spmm_csr_narrow(int32_t rows, int32_t nnz, const int32_t *pos, const int32_t *crd,
                                  const float *vals, const float *B, int32_t k, int64_t ldb, float *C, int64_t ldc,
                                  int32_t tile, const Workspace &w, hipStream_t s);
hipError_t launch_spmm_rowsplit(int32_t rows, const int32_t *pos, const int32_t *crd, const float *vals,
                                const float *B, int32_t k, int64_t ldb, float *C, int64_t ldc,
                                hipStream_t s);

// BCSR (SpMV: bs = 4 has its own kernel, 2 and 8 share one; SpMM: bs in {2, 4, 8})
bool bcsr_tile_ok(int32_t tile);
bool bcsr_g_tile_ok(int32_t bs, int32_t tile);
hipError_t launch_spmv_bcsr_g_main(int32_t bs, int32_t brows, int32_t nblocks, const int32_t *pos, const int32_t *crd,
                                   const float *vals, const float *x, float *y, int32_t tile, const Workspace &w,
                                   hipStream_t s);
hipError_t launch_spmv_bcsr4_main(int32_t brows, int32_t nblocks, const int32_t *pos, const int32_t *crd,
                                  const float *vals, const float *x, float *y, int32_t tile,
                                  const Workspace &w, hipStream_t s);
hipError_t launch_spmm_bcsr_main(int32_t bs, int32_t brows, int32_t nblocks, const int32_t *pos, const int32_t *crd,
                                  const float *vals, const float *B, int32_t k, int64_t ldb, float *C,
                                  int64_t ldc, int32_t tile, const Workspace &w, hipStream_t s);

// Column-slab hierarchy of a CSR matrix (slab.hip)
constexpr int32_t kSlabCols = 32736;        // columns per slab: 32 * 1023 floats = 127.9 KB of x in LDS (15-bit in-slab column)
constexpr int32_t kSlabColsF64 = 16352;     // fp64: 127.75 KB of x next to 32 KB of pair sums (8 waves x 512 doubles)
constexpr int32_t kSlabWavesF64 = 8;
constexpr int32_t kSlabChunk = 512;         // slots per chunk (one wave: 8 per lane)
constexpr int32_t kSlabBuildBlock = 2048;   // CSR positions per block of the bucketing kernels
constexpr int32_t kSlabMaxSlabs = 8192;     // the bucketing kernels keep one counter per slab in LDS
constexpr int32_t kSlabTile = 2048;         // position tile of the second step (pairs per workgroup)
constexpr int32_t kSlabTileF64 = 1024;      // the same for fp64 (its tile kernel holds twice the LDS per position)
inline int64_t slab_max_slots(int64_t cols, int64_t nnz, int32_t W)
{
    const int64_t S = (cols + W - 1) / W;
    const int64_t padded = nnz + S * (kSlabChunk - 1);
    return (padded + kSlabChunk - 1) / kSlabChunk * kSlabChunk;
}
struct SlabBuildSpace {
    int32_t *meta, *tile_row, *H, *srow, *src, *F, *mark, *pair_at, *scan_tmp;
    size_t bytes;
};
size_t scan_tmp_ints(int64_t n);
SlabBuildSpace carve_slab_build(void *base, int64_t rows, int64_t cols, int64_t nnz, int32_t W);
hipError_t launch_slab_build(int32_t rows, int32_t cols, int32_t nnz, const int32_t *pos, const int32_t *crd,
                             const float *vals, const SlabBuildSpace &w, float *svals, uint16_t *scol,
                             int32_t *chunk_pair, int32_t *slab_chunk, int32_t *qpos, int32_t *qidx, hipStream_t s);
hipError_t launch_slab_build_f64(int32_t rows, int32_t cols, int32_t nnz, const int32_t *pos, const int32_t *crd,
                                 const double *vals, const SlabBuildSpace &w, double *svals, uint16_t *scol,
                                 int32_t *chunk_pair, int32_t *slab_chunk, int32_t *qpos, int32_t *qidx, hipStream_t s);
hipError_t launch_slab_pairs_f64(const double *svals, const uint16_t *scol, const int32_t *chunk_pair,
                                 const int32_t *slab_chunk, const double *x, double *P, int32_t cols, int32_t nslabs,
                                 int32_t nchunks, int32_t nwg, int32_t *gap, hipStream_t s);
hipError_t launch_slab_pairs(const float *svals, const uint16_t *scol, const int32_t *chunk_pair,
                             const int32_t *slab_chunk, const float *x, float *P, int32_t cols, int32_t nslabs,
                             int32_t nchunks, int32_t nwg, int32_t *gap, hipStream_t s);
hipError_t launch_fill_int(int32_t *p, int64_t n, int32_t v, hipStream_t s);
// y = Q * P with unit values: the tile kernel of the CSR SpMV without the load of vals (tile 2048)
hipError_t launch_spmv_csr_ones(int32_t rows, int32_t cols, int32_t nnz, const int32_t *pos, const int32_t *crd,
                                const float *x, float *y, const Workspace &w, hipStream_t s);
hipError_t launch_spmv_csr_f64_ones(int32_t rows, int32_t nnz, const int32_t *pos, const int32_t *crd, const double *x,
                                    double *y, int32_t tile, const Workspace &w, hipStream_t s);

#ifdef PSK_CU_TRACE
hipError_t cu_trace_set_spmv_csr(void *buf, unsigned records);
hipError_t cu_trace_set_slab(void *buf, unsigned records);
#endif

// MTTKRP on a three-level hierarchy
bool mttkrp_tile_ok(int32_t tile);
hipError_t launch_partition_csf3(int32_t nslices, int32_t nfibers, int32_t nnz, const int32_t *pos_k,
                                 const int32_t *pos_l, int32_t tile, int32_t *tile_slice, int32_t *tile_fiber,
                                 hipStream_t s);
hipError_t launch_mttkrp_main(int32_t nslices, int32_t nnz, const int32_t *crd_i, const int32_t *pos_k,
                              const int32_t *crd_k, const int32_t *pos_l, const int32_t *crd_l, const float *vals,
                              const float *C, int64_t ldc, const float *D, int64_t ldd, int32_t j, float *A,
                              int64_t lda, int32_t tile, const Workspace &w, const int32_t *tile_fiber,
                              hipStream_t s);

}  // namespace psk
