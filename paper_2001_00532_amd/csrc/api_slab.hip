// C-ABI layer of the column-slab hierarchy: sizes, the analysis step, the product.  No kernels here.
#include "../../include/psk.h"
#include "psk_internal.h"

using namespace psk;

namespace {

constexpr int64_t kMaxI32 = 2147483647ll;

inline int hip_status(hipError_t e) { return e == hipSuccess ? PSK_OK : PSK_ERR_HIP; }

struct SlabMem {
    float *svals;
    uint16_t *scol;
    int32_t *chunk_pair, *slab_chunk, *qpos, *qidx, *qtile_row;
    size_t bytes;
};

SlabMem carve_slab_mem(void *base, int64_t rows, int64_t cols, int64_t nnz)
{
    SlabMem m;
    const int64_t S = (cols + kSlabCols - 1) / kSlabCols;
    const int64_t nmax = slab_max_slots(cols, nnz);
    char *p = static_cast<char *>(base);
    size_t o = 0;
    auto take = [&](size_t bytes) { char *q = p + o; o += align256(bytes); return q; };
    m.svals = reinterpret_cast<float *>(take((size_t)nmax * 4));
    m.scol = reinterpret_cast<uint16_t *>(take((size_t)nmax * 2));
    m.chunk_pair = reinterpret_cast<int32_t *>(take((size_t)(nmax / kSlabChunk + 1) * 4));
    m.slab_chunk = reinterpret_cast<int32_t *>(take((size_t)(S + 1) * 4));
    m.qpos = reinterpret_cast<int32_t *>(take((size_t)(rows + 1) * 4));
    m.qidx = reinterpret_cast<int32_t *>(take((size_t)(nnz + 1) * 4));                     // at most one listed pair per entry
    m.qtile_row = reinterpret_cast<int32_t *>(take((size_t)(nnz / kSlabTile + 2) * 4));
    m.bytes = o;
    return m;
}

// rows, cols, nnz that the slab path accepts
int check_sizes(int64_t rows, int64_t cols, int64_t nnz)
{
    if (rows < 0 || cols < 0 || nnz < 0 || nnz > kMaxI32 || rows > kMaxI32 - 1 || cols > kMaxI32) return PSK_ERR_SIZE;
    if (nnz > 0 && (rows == 0 || cols == 0)) return PSK_ERR_SIZE;
    const int64_t S = (cols + kSlabCols - 1) / kSlabCols;
    if (S > kSlabMaxSlabs) return PSK_ERR_UNSUPPORTED;
    if (slab_max_slots(cols, nnz) > kMaxI32 - 1) return PSK_ERR_SIZE;
    const int64_t nblk = (nnz + kSlabBuildBlock - 1) / kSlabBuildBlock;
    if (S * nblk > (int64_t(1) << 30)) return PSK_ERR_UNSUPPORTED;
    return PSK_OK;
}

}  // namespace

extern "C" {

size_t psk_slab_mem_bytes(int64_t rows, int64_t cols, int64_t nnz)
{
    if (check_sizes(rows, cols, nnz) != PSK_OK) return 0;
    return carve_slab_mem(nullptr, rows, cols, nnz).bytes;
}

size_t psk_slab_build_workspace_bytes(int64_t rows, int64_t cols, int64_t nnz)
{
    if (check_sizes(rows, cols, nnz) != PSK_OK) return 0;
    return carve_slab_build(nullptr, rows, cols, nnz).bytes;
}

size_t psk_slab_spmv_workspace_bytes(const psk_slab *S)
{
    if (!S || S->npairs < 0 || S->nq < 0) return 0;
    return align256((size_t)(S->npairs + 1) * 4) + carve(nullptr, psk_num_tiles(S->nq, kSlabTile), 1).bytes;
}

int psk_slab_build_csr(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd,
                       const float *vals, void *mem, size_t mem_bytes, void *workspace, size_t workspace_bytes,
                       psk_slab *out, void *stream)
{
    int st = check_sizes(rows, cols, nnz);
    if (st != PSK_OK) return st;
    if (!out || !pos || (nnz > 0 && (!crd || !vals))) return PSK_ERR_NULL;
    if (!mem || (reinterpret_cast<uintptr_t>(mem) & 255) || mem_bytes < psk_slab_mem_bytes(rows, cols, nnz))
        return PSK_ERR_WORKSPACE;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) ||
        workspace_bytes < psk_slab_build_workspace_bytes(rows, cols, nnz))
        return PSK_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const SlabMem m = carve_slab_mem(mem, rows, cols, nnz);
    const SlabBuildSpace w = carve_slab_build(workspace, rows, cols, nnz);
    const int64_t S = (cols + kSlabCols - 1) / kSlabCols;
    psk_slab d;
    d.rows = rows; d.cols = cols; d.nnz = nnz;
    d.nslabs = S; d.nslots = 0; d.nchunks = 0; d.npairs = 0; d.nq = 0;
    d.slab_cols = kSlabCols; d.chunk = kSlabChunk; d.tile = kSlabTile; d.reserved = 0;
    d.svals = m.svals; d.scol = m.scol; d.chunk_pair = m.chunk_pair; d.slab_chunk = m.slab_chunk;
    d.qpos = m.qpos; d.qidx = m.qidx; d.qtile_row = m.qtile_row;
    hipError_t e = hipSuccess;
    if (nnz == 0) {
        // no slots, no pairs: the tables are all zero and the product only clears y
        e = launch_fill_int(m.slab_chunk, S + 1, 0, s);
        if (e == hipSuccess) e = launch_fill_int(m.chunk_pair, 1, 0, s);
        if (e == hipSuccess) e = launch_fill_int(m.qpos, rows + 1, 0, s);
        if (e == hipSuccess) e = launch_fill_int(m.qtile_row, 1, (int32_t)rows, s);
        if (e == hipSuccess) e = hipStreamSynchronize(s);
        *out = d;
        return hip_status(e);
    }
    e = launch_slab_build((int32_t)rows, (int32_t)cols, (int32_t)nnz, pos, crd, vals, w, m.svals, m.scol, m.chunk_pair,
                          m.slab_chunk, m.qpos, m.qidx, s);
    if (e != hipSuccess) return PSK_ERR_HIP;
    int32_t meta[3] = {0, 0, 0};
    if (hipMemcpyAsync(meta, w.meta, sizeof(meta), hipMemcpyDeviceToHost, s) != hipSuccess) return PSK_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return PSK_ERR_HIP;
    d.nslots = meta[0];
    d.nchunks = meta[0] / kSlabChunk;
    d.npairs = meta[1];
    d.nq = meta[2];
    // the position cut of the row lists, kept with the structure (it depends only on A)
    e = launch_partition(rows, d.nq, m.qpos, kSlabTile, 0, m.qtile_row, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    *out = d;
    return hip_status(e);
}

int psk_spmv_slab(const psk_slab *S, const float *x, float *y, int phases, void *workspace, size_t workspace_bytes,
                  void *stream)
{
    if (!S) return PSK_ERR_NULL;
    if (phases <= 0 || (phases & ~PSK_PHASE_ALL)) return PSK_ERR_UNSUPPORTED;
    if (S->rows < 0 || S->cols < 0 || S->nnz < 0 || S->npairs < 0 || S->nq < 0 || S->nchunks < 0 ||
        S->slab_cols != kSlabCols || S->chunk != kSlabChunk || S->tile != kSlabTile)
        return PSK_ERR_SIZE;
    if ((S->rows > 0 && !y) || (S->nnz > 0 && !x)) return PSK_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (S->nnz == 0) return hip_status((phases & PSK_PHASE_MAIN) ? launch_fill_zero(y, S->rows, s) : hipSuccess);
    if (!S->svals || !S->scol || !S->chunk_pair || !S->slab_chunk || !S->qpos || !S->qidx || !S->qtile_row)
        return PSK_ERR_NULL;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) ||
        workspace_bytes < psk_slab_spmv_workspace_bytes(S))
        return PSK_ERR_WORKSPACE;
    float *P = static_cast<float *>(workspace);
    const size_t p_bytes = align256((size_t)(S->npairs + 1) * 4);
    const int32_t ntiles = (int32_t)psk_num_tiles(S->nq, kSlabTile);
    Workspace ws = carve(static_cast<char *>(workspace) + p_bytes, ntiles, 1);
    ws.tile_row = const_cast<int32_t *>(S->qtile_row);         // the table is part of the structure; only read
    // step 1: one persistent workgroup per compute unit (a workgroup holds 128 KB of the CU's LDS)
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) cus = v;
    }
    hipError_t e = hipSuccess;
    if (phases & PSK_PHASE_MAIN) {
        e = launch_slab_pairs(S->svals, S->scol, S->chunk_pair, S->slab_chunk, x, P, (int32_t)S->cols,
                              (int32_t)S->nslabs, (int32_t)S->nchunks, cus, ws.gap, s);
        // step 2: rows add up their pairs (position cut of the row lists, carries)
        if (e == hipSuccess) {
            if (ntiles == 0) e = launch_fill_zero(y, S->rows, s);
            else e = launch_spmv_csr_ones((int32_t)S->rows, (int32_t)S->npairs, (int32_t)S->nq, S->qpos, S->qidx, P, y, ws, s);
        }
    }
    if ((phases & PSK_PHASE_FIXUP) && e == hipSuccess)
        e = launch_carry_fixup(ntiles, 1, 1, 1, kSlabTile, S->qpos, ws, y, s, nullptr, nullptr, true);
    return hip_status(e);
}

}  // extern "C"
