// C-ABI layer of the column-slab hierarchy: sizes, the analysis step, the product.  No kernels here.
#include "../../include/psk.h"
#include "psk_internal.h"

using namespace psk;

namespace {

constexpr int64_t kMaxI32 = 2147483647ll;

inline int hip_status(hipError_t e) { return e == hipSuccess ? PSK_OK : PSK_ERR_HIP; }

struct SlabMem {
    void *svals;
    uint16_t *scol;
    int32_t *chunk_pair, *slab_chunk, *qpos, *qidx, *qtile_row;
    size_t bytes;
};

// columns per slab for values of vbytes bytes (4: float, 8: double)
inline int32_t slab_w(int vbytes) { return vbytes == 8 ? kSlabColsF64 : kSlabCols; }
// position tile of the row sums
inline int32_t slab_tile(int vbytes) { return vbytes == 8 ? kSlabTileF64 : kSlabTile; }

SlabMem carve_slab_mem(void *base, int64_t rows, int64_t cols, int64_t nnz, int vbytes)
{
    SlabMem m;
    const int32_t W = slab_w(vbytes);
    const int64_t S = (cols + W - 1) / W;
    const int64_t nmax = slab_max_slots(cols, nnz, W);
    char *p = static_cast<char *>(base);
    size_t o = 0;
    auto take = [&](size_t bytes) { char *q = p + o; o += align256(bytes); return q; };
    m.svals = take((size_t)nmax * (size_t)vbytes);
    m.scol = reinterpret_cast<uint16_t *>(take((size_t)nmax * 2));
    m.chunk_pair = reinterpret_cast<int32_t *>(take((size_t)(nmax / kSlabChunk + 1) * 4));
    m.slab_chunk = reinterpret_cast<int32_t *>(take((size_t)(S + 1) * 4));
    m.qpos = reinterpret_cast<int32_t *>(take((size_t)(rows + 1) * 4));
    m.qidx = reinterpret_cast<int32_t *>(take((size_t)(nnz + 1) * 4));                     // at most one listed pair per entry
    m.qtile_row = reinterpret_cast<int32_t *>(take((size_t)(nnz / slab_tile(vbytes) + 2) * 4));
    m.bytes = o;
    return m;
}

// rows, cols, nnz that the slab path accepts
int check_sizes(int64_t rows, int64_t cols, int64_t nnz, int vbytes)
{
    if (rows < 0 || cols < 0 || nnz < 0 || nnz > kMaxI32 || rows > kMaxI32 - 1 || cols > kMaxI32) return PSK_ERR_SIZE;
    if (nnz > 0 && (rows == 0 || cols == 0)) return PSK_ERR_SIZE;
    const int32_t W = slab_w(vbytes);
    const int64_t S = (cols + W - 1) / W;
    if (S > kSlabMaxSlabs) return PSK_ERR_UNSUPPORTED;
    if (slab_max_slots(cols, nnz, W) > kMaxI32 - 1) return PSK_ERR_SIZE;
    const int64_t nblk = (nnz + kSlabBuildBlock - 1) / kSlabBuildBlock;
    if (S * nblk > (int64_t(1) << 30)) return PSK_ERR_UNSUPPORTED;
    return PSK_OK;
}

size_t mem_bytes(int64_t rows, int64_t cols, int64_t nnz, int vbytes)
{
    if (check_sizes(rows, cols, nnz, vbytes) != PSK_OK) return 0;
    return carve_slab_mem(nullptr, rows, cols, nnz, vbytes).bytes;
}

size_t build_workspace_bytes(int64_t rows, int64_t cols, int64_t nnz, int vbytes)
{
    if (check_sizes(rows, cols, nnz, vbytes) != PSK_OK) return 0;
    return carve_slab_build(nullptr, rows, cols, nnz, slab_w(vbytes)).bytes;
}

int build_csr(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd, const void *vals,
              int vbytes, void *mem, size_t mem_size, void *workspace, size_t workspace_bytes, psk_slab *out,
              void *stream)
{
    int st = check_sizes(rows, cols, nnz, vbytes);
    if (st != PSK_OK) return st;
    if (!out || !pos || (nnz > 0 && (!crd || !vals))) return PSK_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(vals) & (uintptr_t)(vbytes - 1)) return PSK_ERR_ALIGNMENT;
    if (!mem || (reinterpret_cast<uintptr_t>(mem) & 255) || mem_size < mem_bytes(rows, cols, nnz, vbytes))
        return PSK_ERR_WORKSPACE;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) ||
        workspace_bytes < build_workspace_bytes(rows, cols, nnz, vbytes))
        return PSK_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int32_t W = slab_w(vbytes);
    const SlabMem m = carve_slab_mem(mem, rows, cols, nnz, vbytes);
    const SlabBuildSpace w = carve_slab_build(workspace, rows, cols, nnz, W);
    const int64_t S = (cols + W - 1) / W;
    psk_slab d;
    d.rows = rows; d.cols = cols; d.nnz = nnz;
    d.nslabs = S; d.nslots = 0; d.nchunks = 0; d.npairs = 0; d.nq = 0;
    d.slab_cols = W; d.chunk = kSlabChunk; d.tile = slab_tile(vbytes); d.value_bytes = vbytes;
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
    if (vbytes == 8)
        e = launch_slab_build_f64((int32_t)rows, (int32_t)cols, (int32_t)nnz, pos, crd, static_cast<const double *>(vals), w,
                                  static_cast<double *>(m.svals), m.scol, m.chunk_pair, m.slab_chunk, m.qpos, m.qidx, s);
    else
        e = launch_slab_build((int32_t)rows, (int32_t)cols, (int32_t)nnz, pos, crd, static_cast<const float *>(vals), w,
                              static_cast<float *>(m.svals), m.scol, m.chunk_pair, m.slab_chunk, m.qpos, m.qidx, s);
    if (e != hipSuccess) return PSK_ERR_HIP;
    int32_t meta[3] = {0, 0, 0};
    if (hipMemcpyAsync(meta, w.meta, sizeof(meta), hipMemcpyDeviceToHost, s) != hipSuccess) return PSK_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return PSK_ERR_HIP;
    d.nslots = meta[0];
    d.nchunks = meta[0] / kSlabChunk;
    d.npairs = meta[1];
    d.nq = meta[2];
    // the position cut of the row lists, kept with the structure (it depends only on A)
    e = launch_partition(rows, d.nq, m.qpos, slab_tile(vbytes), 0, m.qtile_row, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    *out = d;
    return hip_status(e);
}

int spmv_slab(const psk_slab *S, const void *x, void *y, int vbytes, int phases, void *workspace,
              size_t workspace_bytes, void *stream)
{
    if (!S) return PSK_ERR_NULL;
    if (phases <= 0 || (phases & ~PSK_PHASE_ALL)) return PSK_ERR_UNSUPPORTED;
    if (S->rows < 0 || S->cols < 0 || S->nnz < 0 || S->npairs < 0 || S->nq < 0 || S->nchunks < 0 ||
        S->value_bytes != vbytes || S->slab_cols != slab_w(vbytes) || S->chunk != kSlabChunk || S->tile != slab_tile(vbytes))
        return PSK_ERR_SIZE;
    // the sizes a build leaves are consistent with each other; a struct that is not was not made by psk_slab_build_csr
    if (S->rows > kMaxI32 - 1 || S->cols > kMaxI32 || S->nnz > kMaxI32 || S->nslots > kMaxI32 ||
        S->nslabs != (S->cols + S->slab_cols - 1) / S->slab_cols || S->nslots != S->nchunks * kSlabChunk ||
        S->nslots < S->nnz || S->nslots > slab_max_slots(S->cols, S->nnz, S->slab_cols) || S->npairs > S->nslots ||
        S->nq > S->npairs || S->nq > S->nnz || (S->nnz > 0 && S->npairs < 1))
        return PSK_ERR_SIZE;
    if ((S->rows > 0 && !y) || (S->nnz > 0 && !x)) return PSK_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(y)) & (uintptr_t)(vbytes - 1)) return PSK_ERR_ALIGNMENT;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t zero_words = S->rows * (vbytes / 4);          // +0.0 is all zero bits in either type
    if (S->nnz == 0)
        return hip_status((phases & PSK_PHASE_MAIN) ? launch_fill_zero(static_cast<float *>(y), zero_words, s) : hipSuccess);
    if (!S->svals || !S->scol || !S->chunk_pair || !S->slab_chunk || !S->qpos || !S->qidx || !S->qtile_row)
        return PSK_ERR_NULL;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) ||
        workspace_bytes < psk_slab_spmv_workspace_bytes(S))
        return PSK_ERR_WORKSPACE;
    const size_t p_bytes = align256((size_t)(S->npairs + 1) * (size_t)vbytes);
    const int32_t tile = slab_tile(vbytes);
    const int32_t ntiles = (int32_t)psk_num_tiles(S->nq, tile);
    Workspace ws = carve(static_cast<char *>(workspace) + p_bytes, ntiles, vbytes / 4);
    ws.tile_row = const_cast<int32_t *>(S->qtile_row);         // the table is part of the structure; only read
    // step 1: one persistent workgroup per compute unit (a workgroup holds the CU's LDS)
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) cus = v;
    }
    hipError_t e = hipSuccess;
    if (vbytes == 8) {
        double *P = static_cast<double *>(workspace);
        double *yd = static_cast<double *>(y);
        if (phases & PSK_PHASE_MAIN) {
            e = launch_slab_pairs_f64(static_cast<const double *>(S->svals), S->scol, S->chunk_pair, S->slab_chunk,
                                      static_cast<const double *>(x), P, (int32_t)S->cols, (int32_t)S->nslabs,
                                      (int32_t)S->nchunks, cus, ws.gap, s);
            if (e == hipSuccess) {
                if (ntiles == 0) e = launch_fill_zero(static_cast<float *>(y), zero_words, s);
                else e = launch_spmv_csr_f64_ones((int32_t)S->rows, (int32_t)S->nq, S->qpos, S->qidx, P, yd, tile, ws, s);
            }
        }
        if ((phases & PSK_PHASE_FIXUP) && e == hipSuccess) e = launch_carry_fixup_f64(ntiles, tile, S->qpos, ws, yd, s, true);
        return hip_status(e);
    }
    float *P = static_cast<float *>(workspace);
    float *yf = static_cast<float *>(y);
    if (phases & PSK_PHASE_MAIN) {
        e = launch_slab_pairs(static_cast<const float *>(S->svals), S->scol, S->chunk_pair, S->slab_chunk,
                              static_cast<const float *>(x), P, (int32_t)S->cols, (int32_t)S->nslabs,
                              (int32_t)S->nchunks, cus, ws.gap, s);
        // step 2: rows add up their pairs (position cut of the row lists, carries)
        if (e == hipSuccess) {
            if (ntiles == 0) e = launch_fill_zero(yf, S->rows, s);
            else e = launch_spmv_csr_ones((int32_t)S->rows, (int32_t)S->npairs, (int32_t)S->nq, S->qpos, S->qidx, P, yf, ws, s);
        }
    }
    if ((phases & PSK_PHASE_FIXUP) && e == hipSuccess)
        e = launch_carry_fixup(ntiles, 1, 1, 1, tile, S->qpos, ws, yf, s, nullptr, nullptr, true);
    return hip_status(e);
}

}  // namespace

extern "C" {

size_t psk_slab_mem_bytes(int64_t rows, int64_t cols, int64_t nnz) { return mem_bytes(rows, cols, nnz, 4); }
size_t psk_slab_mem_bytes_f64(int64_t rows, int64_t cols, int64_t nnz) { return mem_bytes(rows, cols, nnz, 8); }

size_t psk_slab_build_workspace_bytes(int64_t rows, int64_t cols, int64_t nnz)
{
    return build_workspace_bytes(rows, cols, nnz, 4);
}
size_t psk_slab_build_workspace_bytes_f64(int64_t rows, int64_t cols, int64_t nnz)
{
    return build_workspace_bytes(rows, cols, nnz, 8);
}

size_t psk_slab_spmv_workspace_bytes(const psk_slab *S)
{
    if (!S || S->npairs < 0 || S->nq < 0 || (S->value_bytes != 4 && S->value_bytes != 8)) return 0;
    return align256((size_t)(S->npairs + 1) * (size_t)S->value_bytes) +
           carve(nullptr, psk_num_tiles(S->nq, slab_tile(S->value_bytes)), S->value_bytes / 4).bytes;
}

int psk_slab_build_csr(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd,
                       const float *vals, void *mem, size_t mem_bytes_, void *workspace, size_t workspace_bytes,
                       psk_slab *out, void *stream)
{
    return build_csr(rows, cols, nnz, pos, crd, vals, 4, mem, mem_bytes_, workspace, workspace_bytes, out, stream);
}

int psk_slab_build_csr_f64(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd,
                           const double *vals, void *mem, size_t mem_bytes_, void *workspace, size_t workspace_bytes,
                           psk_slab *out, void *stream)
{
    return build_csr(rows, cols, nnz, pos, crd, vals, 8, mem, mem_bytes_, workspace, workspace_bytes, out, stream);
}

int psk_spmv_slab(const psk_slab *S, const float *x, float *y, int phases, void *workspace, size_t workspace_bytes,
                  void *stream)
{
    return spmv_slab(S, x, y, 4, phases, workspace, workspace_bytes, stream);
}

int psk_spmv_slab_f64(const psk_slab *S, const double *x, double *y, int phases, void *workspace,
                      size_t workspace_bytes, void *stream)
{
    return spmv_slab(S, x, y, 8, phases, workspace, workspace_bytes, stream);
}

}  // extern "C"
