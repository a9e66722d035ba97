// C-ABI layer: argument validation, workspace carving, phase dispatch.  No kernels here.
#include "../../include/psk.h"
#include "psk_internal.h"
#include <mutex>

using namespace psk;

namespace psk {
thread_local hipError_t tls_launch_status = hipSuccess;
}

// Scratch memory of psk_spmv_csr_static: one copy per GPU, held until the process ends.  The name is only a
// host-side handle; the device address is asked for once per device (static_scratch()) and that pointer is
// what the kernels receive.
static __device__ __align__(256) unsigned char scratch[PSK_STATIC_SCRATCH_BYTES];

namespace {

constexpr int64_t kMaxI32 = 2147483647ll;

constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void *scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device; NULL (and *err set) when the runtime refuses.
void *static_scratch(hipError_t *err)
{
    int dev = -1;
    *err = hipGetDevice(&dev);
    if (*err != hipSuccess) return nullptr;
    if (dev < 0 || dev >= kMaxDevices) { *err = hipErrorInvalidDevice; return nullptr; }
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void *p = nullptr;
        *err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (*err != hipSuccess || !p) { if (*err == hipSuccess) *err = hipErrorInvalidSymbol; return nullptr; }
        scratch_ptr[dev] = p;
    }
    return scratch_ptr[dev];
}

int32_t default_tile(int op, int32_t bs = 4)
{
    if (op == PSK_OP_SPMV_BCSR && bs == 2) return 1024;
    if (op == PSK_OP_SPMV_BCSR && bs == 8) return 64;
    switch (op) {
        case PSK_OP_SPMV_CSR: return 2048;
        case PSK_OP_SPMM_CSR: return 512;
        case PSK_OP_SPMV_BCSR: return 512;
        case PSK_OP_SPMM_BCSR: return 64;
        case PSK_OP_MTTKRP_CSF3: return 2048;
        case PSK_OP_SPMV_CSR_F64: return 1024;
        default: return -1;
    }
}

bool tile_ok(int op, int32_t tile, int32_t bs = 4)
{
    if (op == PSK_OP_SPMV_BCSR && bs != 4) return bcsr_g_tile_ok(bs, tile);
    switch (op) {
        case PSK_OP_SPMV_CSR: return spmv_csr_tile_ok(tile);
        case PSK_OP_SPMM_CSR: return spmm_csr_tile_ok(tile);
        case PSK_OP_SPMV_BCSR:
        case PSK_OP_SPMM_BCSR: return bcsr_tile_ok(tile);
        case PSK_OP_MTTKRP_CSF3: return mttkrp_tile_ok(tile);
        case PSK_OP_SPMV_CSR_F64: return spmv_csr_f64_tile_ok(tile);
        default: return false;
    }
}

int64_t carry_width(int op, int32_t k, int32_t bs)
{
    switch (op) {
        case PSK_OP_SPMV_CSR: return 1;
        case PSK_OP_SPMM_CSR: return k;
        case PSK_OP_SPMV_BCSR: return bs;
        case PSK_OP_SPMM_BCSR: return (int64_t)bs * k;
        case PSK_OP_MTTKRP_CSF3: return k;
        case PSK_OP_SPMV_CSR_F64: return 2;   // one double per tile
        default: return 0;
    }
}

// Common checks of the sparse operand and the execution arguments.  On success *tile holds the
// effective tile size and *ws the carved workspace.
int check_common(int op, int64_t rows, int64_t cols, int64_t nnz, const void *pos, const void *crd,
                 const void *vals, int32_t k, int32_t bs, int32_t *tile, int phases, void *workspace,
                 size_t workspace_bytes, Workspace *ws)
{
    if (rows < 0 || cols < 0 || nnz < 0 || nnz > kMaxI32 || rows > kMaxI32 - 1 || cols > kMaxI32) return PSK_ERR_SIZE;
    if (nnz > 0 && (rows == 0 || cols == 0)) return PSK_ERR_SIZE;
    if (!pos) return PSK_ERR_NULL;
    if (nnz > 0 && (!crd || !vals)) return PSK_ERR_NULL;
    if (phases <= 0 || (phases & ~PSK_PHASE_ALL)) return PSK_ERR_UNSUPPORTED;
    if (*tile == 0) *tile = default_tile(op, bs);
    if (!tile_ok(op, *tile, bs)) return PSK_ERR_TILE;
    const size_t need = psk_workspace_bytes(op, rows, nnz, k, bs, *tile);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) || workspace_bytes < need) return PSK_ERR_WORKSPACE;
    const int64_t ntiles = psk_num_tiles(nnz, *tile);
    *ws = carve(workspace, ntiles, carry_width(op, k, bs));
    return PSK_OK;
}

inline int hip_status(hipError_t e) { return e == hipSuccess ? PSK_OK : PSK_ERR_HIP; }

}  // namespace

extern "C" {

const char *psk_status_string(int status)
{
    switch (status) {
        case PSK_OK: return "ok";
        case PSK_ERR_NULL: return "a required pointer is NULL";
        case PSK_ERR_SIZE: return "invalid size argument";
        case PSK_ERR_TILE: return "unsupported position-tile size";
        case PSK_ERR_WORKSPACE: return "workspace missing, misaligned or too small (or the problem exceeds the built-in scratch memory)";
        case PSK_ERR_UNSUPPORTED: return "unsupported operation, variant or phase mask";
        case PSK_ERR_HIP: return "HIP runtime error at kernel launch";
        case PSK_ERR_ALIGNMENT: return "operand not 16-byte aligned";
        default: return "unknown status";
    }
}

int psk_version(void) { return 100; }

int32_t psk_default_tile(int op) { return default_tile(op); }

int32_t psk_default_tile_bcsr(int op, int32_t bs)
{
    if ((op != PSK_OP_SPMV_BCSR && op != PSK_OP_SPMM_BCSR) || (bs != 2 && bs != 4 && bs != 8)) return -1;
    return default_tile(op, bs);
}

int64_t psk_num_tiles(int64_t nnz, int32_t tile)
{
    if (tile <= 0) return -1;
    return nnz <= 0 ? 0 : (nnz + tile - 1) / tile;
}

size_t psk_workspace_bytes(int op, int64_t rows, int64_t nnz, int32_t k, int32_t bs, int32_t tile)
{
    (void)rows;
    // CSR SpMV picks 2048, or 1024 with column passes: size for the smaller one, which needs more
    if (tile == 0) tile = op == PSK_OP_SPMV_CSR ? 1024 : default_tile(op, bs);
    if (tile <= 0 || nnz < 0 || nnz > kMaxI32) return 0;
    if ((op == PSK_OP_SPMM_CSR || op == PSK_OP_SPMM_BCSR || op == PSK_OP_MTTKRP_CSF3) && k <= 0) return 0;
    if ((op == PSK_OP_SPMV_BCSR || op == PSK_OP_SPMM_BCSR) && bs <= 0) return 0;
    const int64_t width = carry_width(op, k, bs);
    if (width <= 0) return 0;
    return carve(nullptr, psk_num_tiles(nnz, tile), width).bytes;
}

int psk_partition_csr(int64_t rows, int64_t nnz, const int32_t *pos, int32_t tile, int method,
                      int32_t *tile_row, void *stream)
{
    if (rows < 0 || nnz < 0 || nnz > kMaxI32 || rows > kMaxI32 - 1) return PSK_ERR_SIZE;
    if (tile <= 0) return PSK_ERR_TILE;
    if (method < PSK_PARTITION_AUTO || method > PSK_PARTITION_SCAN) return PSK_ERR_UNSUPPORTED;
    if (!pos || !tile_row) return PSK_ERR_NULL;
    return hip_status(launch_partition(rows, nnz, pos, tile, method, tile_row, static_cast<hipStream_t>(stream)));
}

int psk_analyze_csr(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd,
                    void *workspace, size_t workspace_bytes, int32_t *col_passes, void *stream)
{
    if (rows < 0 || cols < 0 || nnz < 0 || nnz > kMaxI32 || rows > kMaxI32 - 1 || cols > kMaxI32) return PSK_ERR_SIZE;
    if (!col_passes || !pos || (nnz > 0 && !crd)) return PSK_ERR_NULL;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) || workspace_bytes < 256) return PSK_ERR_WORKSPACE;
    *col_passes = 1;
    const int64_t x_bytes = cols * 4;
    // x fits the 4 MB L2 of a die (with room for the streams), or the problem is too small to matter
    if (x_bytes <= (int64_t(6) << 20) || nnz < (int64_t(1) << 20)) return PSK_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int32_t *dev = static_cast<int32_t *>(workspace);
    int32_t host[2] = {0, 0};
    if (launch_probe_locality((int32_t)nnz, crd, dev, s) != hipSuccess) return PSK_ERR_HIP;
    if (hipMemcpyAsync(host, dev, sizeof(host), hipMemcpyDeviceToHost, s) != hipSuccess) return PSK_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return PSK_ERR_HIP;
    if (host[1] > 0 && 2 * (int64_t)host[0] < host[1]) {   // fewer than half of the gathers stay in their line
        // slices of up to 6 MiB: measured best at x = 8 MB (2 passes), 16 MB (3) and 32 MB (4, the cap)
        const int64_t want = (x_bytes + (int64_t(6) << 20) - 1) / (int64_t(6) << 20);
        *col_passes = (int32_t)(want > PSK_MAX_COL_PASSES ? PSK_MAX_COL_PASSES : want);
    }
    return PSK_OK;
}

int psk_validate_csr(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd, void *workspace,
                     size_t workspace_bytes, int32_t *violation, void *stream)
{
    if (rows < 0 || cols < 0 || nnz < 0 || nnz > kMaxI32 || rows > kMaxI32 - 1 || cols > kMaxI32) return PSK_ERR_SIZE;
    if (!violation || !pos || (nnz > 0 && !crd)) return PSK_ERR_NULL;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) || workspace_bytes < 256) return PSK_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int32_t *dev = static_cast<int32_t *>(workspace);
    int32_t host[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (launch_validate_csr((int32_t)rows, (int32_t)cols, (int32_t)nnz, pos, crd, dev, s) != hipSuccess) return PSK_ERR_HIP;
    if (hipMemcpyAsync(host, dev, sizeof(host), hipMemcpyDeviceToHost, s) != hipSuccess) return PSK_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return PSK_ERR_HIP;
    *violation = 0;
    for (int c = 1; c <= 4; ++c)
        if (host[c] != 0) { *violation = c; break; }
    return PSK_OK;
}

int psk_suggest_schedule_csr(int64_t rows, int64_t nnz, const int32_t *pos, void *workspace, size_t workspace_bytes,
                             int32_t *schedule, void *stream)
{
    if (rows < 0 || nnz < 0 || nnz > kMaxI32 || rows > kMaxI32 - 1) return PSK_ERR_SIZE;
    if (!schedule || !pos) return PSK_ERR_NULL;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) || workspace_bytes < 256) return PSK_ERR_WORKSPACE;
    *schedule = PSK_SCHEDULE_POSITIONS;
    // Row-split can only win where the two extra launches of the position path are a visible share of
    // the time (small problems) and the rows fill a wave (long enough, and alike).
    if (rows == 0 || nnz > (int64_t(6) << 20) || nnz < 48 * rows) return PSK_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int32_t *dev = static_cast<int32_t *>(workspace);
    int32_t longest = 0;
    if (launch_max_row((int32_t)rows, pos, dev, s) != hipSuccess) return PSK_ERR_HIP;
    if (hipMemcpyAsync(&longest, dev, sizeof(longest), hipMemcpyDeviceToHost, s) != hipSuccess) return PSK_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return PSK_ERR_HIP;
    if (2 * (int64_t)longest * rows <= 7 * nnz) *schedule = PSK_SCHEDULE_ROWS;   // longest <= 3.5 x mean
    return PSK_OK;
}

int psk_spmv_csr(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd,
                 const float *vals, const float *x, float *y, int32_t tile, int32_t col_passes, int phases,
                 void *workspace, size_t workspace_bytes, void *stream)
{
    if (col_passes < 0 || col_passes > PSK_MAX_COL_PASSES) return PSK_ERR_SIZE;
    // a matrix of a few thousand entries is bound by launch latency: with the default tile it is taken as ONE tile
    // by one workgroup -- no table, no carries, one launch instead of three
    const bool single = tile == 0 && col_passes <= 1 && nnz > 0 && nnz <= kSingleTile && rows <= 4 * kSingleTile;
    if (tile == 0 && col_passes > 1) tile = 1024;   // gather-bound passes prefer the smaller tile (measured)
    Workspace ws;
    int st = check_common(PSK_OP_SPMV_CSR, rows, cols, nnz, pos, crd, vals, 1, 1, &tile, phases, workspace,
                          workspace_bytes, &ws);
    if (st != PSK_OK) return st;
    if ((rows > 0 && !y) || (nnz > 0 && !x)) return PSK_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (single) {
        if (!(phases & PSK_PHASE_MAIN)) return PSK_OK;
        return hip_status(launch_spmv_csr_single((int32_t)rows, (int32_t)cols, (int32_t)nnz, pos, crd, vals, x, y, s));
    }
    const int32_t ntiles = (int32_t)psk_num_tiles(nnz, tile);
    hipError_t e = hipSuccess;
    // long runs of empty rows: the tile that spans one lists it (ws.gap) and the fix-up step clears it at full width
    if ((phases & PSK_PHASE_PARTITION) && e == hipSuccess) e = launch_partition(rows, nnz, pos, tile, 0, ws.tile_row, s, ws.gap);
    if ((phases & PSK_PHASE_MAIN) && e == hipSuccess) {
        if (ntiles == 0) e = launch_fill_zero(y, rows, s);
        else e = launch_spmv_csr_main((int32_t)rows, (int32_t)cols, (int32_t)nnz, pos, crd, vals, x, y, tile, col_passes, ws, s,
                                      nullptr, true);
    }
    if ((phases & PSK_PHASE_FIXUP) && e == hipSuccess)
        e = launch_carry_fixup(ntiles, 1, 1, 1, tile, pos, ws, y, s, nullptr, nullptr, true);
    return hip_status(e);
}

int psk_cu_trace_set(void *records, size_t nrecords)
{
#ifdef PSK_CU_TRACE
    if (nrecords > 0xffffffffu) return PSK_ERR_SIZE;
    // the slab pair kernel (persistent, at most PSK_CU_TRACE_SLAB_RECORDS workgroups) records into the first part
    // of the buffer, the CSR kernels behind it, so that a slab product (both kinds of kernel) can be traced at once
    if (records && nrecords <= PSK_CU_TRACE_SLAB_RECORDS) return PSK_ERR_SIZE;
    unsigned long long *base = static_cast<unsigned long long *>(records);
    const unsigned n = records ? (unsigned)(nrecords - PSK_CU_TRACE_SLAB_RECORDS) : 0u;
    if (cu_trace_set_slab(base, records ? PSK_CU_TRACE_SLAB_RECORDS : 0u) != hipSuccess) return PSK_ERR_HIP;
    if (cu_trace_set_spmv_csr(records ? base + 3ull * PSK_CU_TRACE_SLAB_RECORDS : nullptr, n) != hipSuccess) return PSK_ERR_HIP;
    return PSK_OK;
#else
    (void)records;
    (void)nrecords;
    return PSK_ERR_UNSUPPORTED;     // this is the plain build; the instrumented one is libpsk_trace.so
#endif
}

size_t psk_static_scratch_bytes(void) { return PSK_STATIC_SCRATCH_BYTES; }

int psk_spmv_csr_static(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd,
                        const float *vals, const float *x, float *y, int32_t tile, int32_t col_passes, void *stream)
{
    if (col_passes < 0 || col_passes > PSK_MAX_COL_PASSES) return PSK_ERR_SIZE;
    if (tile == 0) tile = col_passes > 1 ? 1024 : default_tile(PSK_OP_SPMV_CSR);
    if (!tile_ok(PSK_OP_SPMV_CSR, tile)) return PSK_ERR_TILE;
    if (nnz >= 0 && nnz <= kMaxI32 &&
        psk_workspace_bytes(PSK_OP_SPMV_CSR, rows, nnz, 1, 1, tile) > (size_t)PSK_STATIC_SCRATCH_BYTES)
        return PSK_ERR_WORKSPACE;               // more tiles than the built-in scratch memory has room for
    // validate before touching the runtime, with a stand-in workspace address that is never dereferenced
    Workspace ws;
    int st = check_common(PSK_OP_SPMV_CSR, rows, cols, nnz, pos, crd, vals, 1, 1, &tile, PSK_PHASE_ALL,
                          reinterpret_cast<void *>(uintptr_t(256)), PSK_STATIC_SCRATCH_BYTES, &ws);
    if (st != PSK_OK) return st;
    if ((rows > 0 && !y) || (nnz > 0 && !x)) return PSK_ERR_NULL;
    hipError_t e = hipSuccess;
    void *base = static_scratch(&e);
    if (!base) return PSK_ERR_HIP;
    // every part of the scratch memory that a product reads is written earlier in the same product (table by
    // the partition, carry records and column ranges by the tile kernel), so nothing needs clearing
    return psk_spmv_csr(rows, cols, nnz, pos, crd, vals, x, y, tile, col_passes, PSK_PHASE_ALL, base,
                        PSK_STATIC_SCRATCH_BYTES, stream);
}

int psk_spmv_csr_f64(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd,
                     const double *vals, const double *x, double *y, int32_t tile, int32_t col_passes, int phases,
                     void *workspace, size_t workspace_bytes, void *stream)
{
    if (col_passes < 0 || col_passes > PSK_MAX_COL_PASSES) return PSK_ERR_SIZE;
    Workspace ws;
    int st = check_common(PSK_OP_SPMV_CSR_F64, rows, cols, nnz, pos, crd, vals, 1, 1, &tile, phases, workspace,
                          workspace_bytes, &ws);
    if (st != PSK_OK) return st;
    if ((rows > 0 && !y) || (nnz > 0 && !x)) return PSK_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(vals) | reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(y)) & 7)
        return PSK_ERR_ALIGNMENT;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int32_t ntiles = (int32_t)psk_num_tiles(nnz, tile);
    hipError_t e = hipSuccess;
    if ((phases & PSK_PHASE_PARTITION) && e == hipSuccess) e = launch_partition(rows, nnz, pos, tile, 0, ws.tile_row, s, ws.gap);
    if ((phases & PSK_PHASE_MAIN) && e == hipSuccess) {
        if (ntiles == 0) e = launch_fill_zero(reinterpret_cast<float *>(y), 2 * rows, s);
        else e = launch_spmv_csr_f64_main((int32_t)rows, (int32_t)cols, (int32_t)nnz, pos, crd, vals, x, y, tile, col_passes,
                                          ws, s, true);
    }
    if ((phases & PSK_PHASE_FIXUP) && e == hipSuccess) e = launch_carry_fixup_f64(ntiles, tile, pos, ws, y, s, true);
    return hip_status(e);
}

int psk_spmv_dcsr(int64_t rows, int64_t cols, int64_t nstored, int64_t nnz, const int32_t *crd_i, const int32_t *pos,
                  const int32_t *crd, const float *vals, const float *x, float *y, int cut, int32_t tile,
                  int32_t col_passes, int phases, void *workspace, size_t workspace_bytes, void *stream)
{
    if (rows < 0 || rows > kMaxI32 || nstored < 0 || nstored > rows) return PSK_ERR_SIZE;
    if (col_passes < 0 || col_passes > PSK_MAX_COL_PASSES) return PSK_ERR_SIZE;
    if (col_passes == 0) col_passes = 1;
    if (tile == 0 && col_passes > 1) tile = 1024;
    if (cut != PSK_CUT_POSITIONS && cut != PSK_CUT_ROWS) return PSK_ERR_UNSUPPORTED;
    if (nstored > 0 && !crd_i) return PSK_ERR_NULL;
    Workspace ws;
    int st = check_common(PSK_OP_SPMV_CSR, nstored, cols, nnz, pos, crd, vals, 1, 1, &tile, phases, workspace,
                          workspace_bytes, &ws);
    if (st != PSK_OK) return st;
    if ((rows > 0 && !y) || (nnz > 0 && !x)) return PSK_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int32_t ntiles = (int32_t)psk_num_tiles(nnz, tile);
    hipError_t e = hipSuccess;
    if (cut == PSK_CUT_ROWS) {
        // tiles of four stored rows, one wave each: no row is divided, so there is no table and no carry
        if (phases & PSK_PHASE_MAIN) {
            e = launch_fill_zero(y, rows, s);
            if (e == hipSuccess)
                e = launch_spmv_rowsplit((int32_t)nstored, pos, crd, vals, x, y, PSK_ROWSPLIT_WAVE_PER_ROW, s, crd_i);
        }
        return hip_status(e);
    }
    if ((phases & PSK_PHASE_PARTITION) && e == hipSuccess) e = launch_partition(nstored, nnz, pos, tile, 0, ws.tile_row, s);
    if ((phases & PSK_PHASE_MAIN) && e == hipSuccess) {
        e = launch_fill_zero(y, rows, s);
        if (ntiles > 0 && e == hipSuccess)
            e = launch_spmv_csr_main((int32_t)nstored, (int32_t)cols, (int32_t)nnz, pos, crd, vals, x, y, tile,
                                     col_passes, ws, s, crd_i);
    }
    if ((phases & PSK_PHASE_FIXUP) && e == hipSuccess && ntiles > 0)
        e = launch_carry_fixup(ntiles, 1, 1, 1, tile, pos, ws, y, s, nullptr, crd_i);
    return hip_status(e);
}

int psk_spmv_csr_divide(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd,
                        const float *vals, const float *x, float *y, int32_t parts, int phases, void *workspace,
                        size_t workspace_bytes, void *stream)
{
    if (parts < 0 || rows > kMaxI32 - 4096) return PSK_ERR_SIZE;
    int32_t tile = kDivideChunk;
    Workspace ws;
    int st = check_common(PSK_OP_SPMV_CSR, rows, cols, nnz, pos, crd, vals, 1, 1, &tile, phases, workspace,
                          workspace_bytes, &ws);
    if (st != PSK_OK) return st;
    if ((rows > 0 && !y) || (nnz > 0 && !x)) return PSK_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t nchunks = psk_num_tiles(nnz, tile);
    if (parts == 0) parts = 2048;                       // eight resident workgroups on each of the 256 CUs
    const int64_t cpp = nchunks == 0 ? 1 : (nchunks + parts - 1) / parts;
    const int32_t nparts = (int32_t)((nchunks + cpp - 1) / cpp);
    hipError_t e = hipSuccess;
    if (phases & PSK_PHASE_MAIN) {
        if (nparts == 0) e = launch_fill_zero(y, rows, s);
        else e = launch_spmv_csr_divide((int32_t)rows, (int32_t)cols, (int32_t)nnz, pos, crd, vals, x, y, nparts, (int32_t)cpp, ws, s);
    }
    // two or more parts: cpp < nchunks, hence cpp * tile < nnz <= 2^31 - 1 (one part has no carries to add)
    const int64_t part_len = cpp * (int64_t)tile;
    if ((phases & PSK_PHASE_FIXUP) && e == hipSuccess && nparts > 1 && part_len <= kMaxI32)
        e = launch_carry_fixup(nparts, 1, 1, 1, (int32_t)part_len, pos, ws, y, s);
    return hip_status(e);
}

int psk_spmv_csr_atomics(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd,
                         const float *vals, const float *x, float *y, int32_t tile, int phases, void *workspace,
                         size_t workspace_bytes, void *stream)
{
    Workspace ws;
    int st = check_common(PSK_OP_SPMV_CSR, rows, cols, nnz, pos, crd, vals, 1, 1, &tile, phases, workspace,
                          workspace_bytes, &ws);
    if (st != PSK_OK) return st;
    if ((rows > 0 && !y) || (nnz > 0 && !x)) return PSK_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int32_t ntiles = (int32_t)psk_num_tiles(nnz, tile);
    hipError_t e = hipSuccess;
    if ((phases & PSK_PHASE_PARTITION) && e == hipSuccess) e = launch_partition(rows, nnz, pos, tile, 0, ws.tile_row, s);
    if ((phases & PSK_PHASE_MAIN) && e == hipSuccess) {
        e = launch_fill_zero(y, rows, s);
        if (ntiles > 0 && e == hipSuccess)
            e = launch_spmv_csr_main((int32_t)rows, (int32_t)cols, (int32_t)nnz, pos, crd, vals, x, y, tile, -1, ws, s);
    }
    return hip_status(e);
}

int psk_spmv_csr_notemp(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd,
                        const float *vals, const float *x, float *y, int32_t tile, int phases, void *workspace,
                        size_t workspace_bytes, void *stream)
{
    Workspace ws;
    int st = check_common(PSK_OP_SPMV_CSR, rows, cols, nnz, pos, crd, vals, 1, 1, &tile, phases, workspace,
                          workspace_bytes, &ws);
    if (st != PSK_OK) return st;
    if ((rows > 0 && !y) || (nnz > 0 && !x)) return PSK_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int32_t ntiles = (int32_t)psk_num_tiles(nnz, tile);
    hipError_t e = hipSuccess;
    if ((phases & PSK_PHASE_PARTITION) && e == hipSuccess) e = launch_partition(rows, nnz, pos, tile, 0, ws.tile_row, s);
    if ((phases & PSK_PHASE_MAIN) && e == hipSuccess) {
        if (ntiles == 0) e = launch_fill_zero(y, rows, s);
        else e = launch_spmv_csr_main((int32_t)rows, (int32_t)cols, (int32_t)nnz, pos, crd, vals, x, y, tile, -2, ws, s);
    }
    if ((phases & PSK_PHASE_FIXUP) && e == hipSuccess && ntiles > 0)
        e = launch_carry_fixup(ntiles, 1, 1, 1, tile, pos, ws, y, s);
    return hip_status(e);
}

int psk_spmm_csr(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd,
                 const float *vals, const float *B, int32_t k, int64_t ldb, float *C, int64_t ldc,
                 int32_t tile, int phases, void *workspace, size_t workspace_bytes, void *stream)
{
    if (k <= 0 || ldb < k || ldc < k) return PSK_ERR_SIZE;
    Workspace ws;
    int st = check_common(PSK_OP_SPMM_CSR, rows, cols, nnz, pos, crd, vals, k, 1, &tile, phases, workspace,
                          workspace_bytes, &ws);
    if (st != PSK_OK) return st;
    if ((rows > 0 && !C) || (nnz > 0 && !B)) return PSK_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int32_t ntiles = (int32_t)psk_num_tiles(nnz, tile);
    hipError_t e = hipSuccess;
    if ((phases & PSK_PHASE_PARTITION) && e == hipSuccess) e = launch_partition(rows, nnz, pos, tile, 0, ws.tile_row, s);
    if ((phases & PSK_PHASE_MAIN) && e == hipSuccess) {
        if (ntiles == 0) {
            e = launch_fill_zero_2d(C, rows, k, ldc, s);
        } else {
            e = launch_spmm_csr_main((int32_t)rows, (int32_t)nnz, pos, crd, vals, B, k, ldb, C, ldc, tile, ws, s);
        }
    }
    if ((phases & PSK_PHASE_FIXUP) && e == hipSuccess) e = launch_carry_fixup(ntiles, 1, k, ldc, tile, pos, ws, C, s);
    return hip_status(e);
}

int psk_spmv_bcsr(int64_t brows, int64_t bcols, int64_t nblocks, int32_t bs, const int32_t *pos,
                  const int32_t *crd, const float *vals, const float *x, float *y, int32_t tile, int phases,
                  void *workspace, size_t workspace_bytes, void *stream)
{
    if (bs != 2 && bs != 4 && bs != 8) return bs <= 0 ? PSK_ERR_SIZE : PSK_ERR_UNSUPPORTED;
    if (brows > (kMaxI32 - 1) / bs || bcols > kMaxI32 / bs || nblocks > kMaxI32 / (bs * bs)) return PSK_ERR_SIZE;
    Workspace ws;
    int st = check_common(PSK_OP_SPMV_BCSR, brows, bcols, nblocks, pos, crd, vals, 1, bs, &tile, phases,
                          workspace, workspace_bytes, &ws);
    if (st != PSK_OK) return st;
    if ((brows > 0 && !y) || (nblocks > 0 && !x)) return PSK_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(vals) & 15) || (reinterpret_cast<uintptr_t>(x) & (bs == 2 ? 7 : 15)))
        return PSK_ERR_ALIGNMENT;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int32_t ntiles = (int32_t)psk_num_tiles(nblocks, tile);
    hipError_t e = hipSuccess;
    if ((phases & PSK_PHASE_PARTITION) && e == hipSuccess) e = launch_partition(brows, nblocks, pos, tile, 0, ws.tile_row, s);
    if ((phases & PSK_PHASE_MAIN) && e == hipSuccess) {
        if (ntiles == 0) e = launch_fill_zero(y, brows * bs, s);
        else if (bs == 4) e = launch_spmv_bcsr4_main((int32_t)brows, (int32_t)nblocks, pos, crd, vals, x, y, tile, ws, s);
        else e = launch_spmv_bcsr_g_main(bs, (int32_t)brows, (int32_t)nblocks, pos, crd, vals, x, y, tile, ws, s);
    }
    if ((phases & PSK_PHASE_FIXUP) && e == hipSuccess) e = launch_carry_fixup(ntiles, 1, bs, bs, tile, pos, ws, y, s);
    return hip_status(e);
}

int psk_spmm_bcsr(int64_t brows, int64_t bcols, int64_t nblocks, int32_t bs, const int32_t *pos,
                  const int32_t *crd, const float *vals, const float *B, int32_t k, int64_t ldb, float *C,
                  int64_t ldc, int32_t tile, int phases, void *workspace, size_t workspace_bytes, void *stream)
{
    if (bs != 2 && bs != 4 && bs != 8) return bs <= 0 ? PSK_ERR_SIZE : PSK_ERR_UNSUPPORTED;
    if (k <= 0 || ldb < k || ldc < k) return PSK_ERR_SIZE;
    if (brows > (kMaxI32 - 1) / bs || bcols > kMaxI32 / bs || nblocks > kMaxI32 / (bs * bs)) return PSK_ERR_SIZE;
    Workspace ws;
    int st = check_common(PSK_OP_SPMM_BCSR, brows, bcols, nblocks, pos, crd, vals, k, bs, &tile, phases,
                          workspace, workspace_bytes, &ws);
    if (st != PSK_OK) return st;
    if ((brows > 0 && !C) || (nblocks > 0 && !B)) return PSK_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(vals) & 15) return PSK_ERR_ALIGNMENT;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int32_t ntiles = (int32_t)psk_num_tiles(nblocks, tile);
    hipError_t e = hipSuccess;
    if ((phases & PSK_PHASE_PARTITION) && e == hipSuccess) e = launch_partition(brows, nblocks, pos, tile, 0, ws.tile_row, s);
    if ((phases & PSK_PHASE_MAIN) && e == hipSuccess) {
        if (ntiles == 0) {
            e = launch_fill_zero_2d(C, brows * bs, k, ldc, s);
        } else {
            e = launch_spmm_bcsr_main(bs, (int32_t)brows, (int32_t)nblocks, pos, crd, vals, B, k, ldb, C, ldc, tile, ws, s);
        }
    }
    if ((phases & PSK_PHASE_FIXUP) && e == hipSuccess) e = launch_carry_fixup(ntiles, bs, k, ldc, tile, pos, ws, C, s);
    return hip_status(e);
}

int psk_partition_csf3(int64_t nslices, int64_t nfibers, int64_t nnz, const int32_t *pos_k, const int32_t *pos_l,
                       int32_t tile, int32_t *tile_slice, int32_t *tile_fiber, void *stream)
{
    if (nslices < 0 || nfibers < 0 || nnz < 0 || nnz > kMaxI32 || nslices > kMaxI32 - 1 || nfibers > kMaxI32 - 1)
        return PSK_ERR_SIZE;
    if (tile <= 0) return PSK_ERR_TILE;
    if (!pos_k || !pos_l || !tile_slice || !tile_fiber) return PSK_ERR_NULL;
    return hip_status(launch_partition_csf3((int32_t)nslices, (int32_t)nfibers, (int32_t)nnz, pos_k, pos_l, tile,
                                            tile_slice, tile_fiber, static_cast<hipStream_t>(stream)));
}

int psk_mttkrp_csf3(int64_t dim_i, int64_t dim_k, int64_t dim_l, int64_t nslices, int64_t nfibers, int64_t nnz,
                    const int32_t *crd_i, const int32_t *pos_k, const int32_t *crd_k, const int32_t *pos_l,
                    const int32_t *crd_l, const float *vals, const float *C, int64_t ldc, const float *D,
                    int64_t ldd, int32_t j, float *A, int64_t lda, int32_t tile, int phases, void *workspace,
                    size_t workspace_bytes, void *stream)
{
    if (dim_i < 0 || dim_k < 0 || dim_l < 0 || nslices < 0 || nfibers < 0 || nslices > dim_i) return PSK_ERR_SIZE;
    if (dim_i > kMaxI32 - 1 || dim_k > kMaxI32 || dim_l > kMaxI32 || nfibers > kMaxI32 - 1) return PSK_ERR_SIZE;
    if (!crd_i && nslices != dim_i) return PSK_ERR_SIZE;          // dense first level: one slice per i
    if (j <= 0 || ldc < j || ldd < j || lda < j) return PSK_ERR_SIZE;
    if (nnz > 0 && nfibers == 0) return PSK_ERR_SIZE;
    Workspace ws;
    int st = check_common(PSK_OP_MTTKRP_CSF3, nslices, dim_l, nnz, pos_l, crd_l, vals, j, 1, &tile, phases, workspace,
                          workspace_bytes, &ws);
    if (st != PSK_OK) return st;
    if (!pos_k || (nfibers > 0 && !crd_k) || (dim_i > 0 && !A) || (nnz > 0 && (!C || !D))) return PSK_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int32_t ntiles = (int32_t)psk_num_tiles(nnz, tile);
    hipError_t e = hipSuccess;
    if ((phases & PSK_PHASE_PARTITION) && e == hipSuccess)
        e = launch_partition_csf3((int32_t)nslices, (int32_t)nfibers, (int32_t)nnz, pos_k, pos_l, tile, ws.tile_row,
                                  ws.tile_aux, s);
    if ((phases & PSK_PHASE_MAIN) && e == hipSuccess) {
        // a compressed first level leaves rows of A without a slice: clear them all first; so does nnz = 0
        if (crd_i || ntiles == 0) e = launch_fill_zero_2d(A, dim_i, j, lda, s);
        if (ntiles > 0 && e == hipSuccess)
            e = launch_mttkrp_main((int32_t)nslices, (int32_t)nnz, crd_i, pos_k, crd_k, pos_l, crd_l, vals, C, ldc, D,
                                   ldd, j, A, lda, tile, ws, ws.tile_aux, s);
    }
    if ((phases & PSK_PHASE_FIXUP) && e == hipSuccess)
        e = launch_carry_fixup(ntiles, 1, j, lda, tile, pos_k, ws, A, s, pos_l, crd_i);
    return hip_status(e);
}

int psk_spmv_csr_rowsplit(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd,
                          const float *vals, const float *x, float *y, int variant, void *stream)
{
    if (rows < 0 || cols < 0 || nnz < 0 || nnz > kMaxI32 || rows > kMaxI32 - 1) return PSK_ERR_SIZE;
    if (variant != PSK_ROWSPLIT_THREAD_PER_ROW && variant != PSK_ROWSPLIT_WAVE_PER_ROW) return PSK_ERR_UNSUPPORTED;
    if (!pos || (rows > 0 && !y) || (nnz > 0 && (!crd || !vals || !x))) return PSK_ERR_NULL;
    return hip_status(launch_spmv_rowsplit((int32_t)rows, pos, crd, vals, x, y, variant, static_cast<hipStream_t>(stream)));
}

int psk_spmm_csr_rowsplit(int64_t rows, int64_t cols, int64_t nnz, const int32_t *pos, const int32_t *crd,
                          const float *vals, const float *B, int32_t k, int64_t ldb, float *C, int64_t ldc,
                          void *stream)
{
    if (rows < 0 || cols < 0 || nnz < 0 || nnz > kMaxI32 || rows > kMaxI32 - 1) return PSK_ERR_SIZE;
    if (k <= 0 || ldb < k || ldc < k) return PSK_ERR_SIZE;
    if (!pos || (rows > 0 && !C) || (nnz > 0 && (!crd || !vals || !B))) return PSK_ERR_NULL;
    return hip_status(launch_spmm_rowsplit((int32_t)rows, pos, crd, vals, B, k, ldb, C, ldc, static_cast<hipStream_t>(stream)));
}

}  // extern "C"
