// Position-space SpMM for CSR (BS = 1) and BCSR 4x4 (BS = 4), plus the row-split SpMM baseline.
//
// Schedule (appendix "SPMM on a GPU"): the fused (i,j) loop runs over A's positions, split into
// tiles (workgroups) and wave chunks; the dense column index k is split over the 64 lanes of a
// wave; the loop over a wave's positions is innermost.  Generalised from "k = wave width exactly"
// to any k: a lane owns VEC adjacent columns and blockIdx.y walks column chunks of 64*VEC.
#include "psk_dev.h"
#include "psk_internal.h"

namespace psk {

// One workgroup (4 waves) per tile of T positions (T/4 consecutive positions per wave) and per
// column chunk.
//
//  - row ends: sflag[i] = r when position t0+i is the last stored position of row r, else -1
//    (filled from the tile's slice of pos; the tile's metadata lives in LDS).  Empty rows in the
//    tile's write range are zero-filled here.
//  - a wave walks its positions 64 at a time: crd / row-end flags / values are loaded one per lane
//    and broadcast with v_readlane, so the address of the B row is wave-uniform and its load is one
//    contiguous 256*VEC-byte access; U B rows are requested before the first FMA.
//  - a row that ends after at least one earlier row end of the same wave is complete: stored to C.
//    The segment before the first row end of a wave, and the one after the last, go to LDS records;
//    wave 0 chains the records in position order: consecutive open segments belong to the row of the
//    next closed one.  A chain whose row began before the tile becomes the tile's carry record; the
//    open chain at the tile's end is stored by this tile if the row began in it, else carried.
template <int BS, int VEC>
__global__ __launch_bounds__(256) void k_spmm_pos(int rows, int nnz, const int *__restrict__ pos,
                                                  const int *__restrict__ crd,
                                                  const float *__restrict__ vals,
                                                  const float *__restrict__ B, int k, long long ldb,
                                                  float *__restrict__ C, long long ldc,
                                                  const int *__restrict__ tile_row,
                                                  int *__restrict__ carry_row,
                                                  float *__restrict__ carry_val, int ntiles, int T)
{
    constexpr int THREADS = 256, NW = THREADS / WAVE, KW = WAVE * VEC;
    constexpr int U = BS == 1 ? 8 : (BS == 2 ? 4 : (BS == 4 ? 2 : 1));   // positions whose B rows are in flight together
    extern __shared__ int sflag[];                // T ints
    __shared__ float srec[2 * NW][BS][KW];
    __shared__ int srec_row[2 * NW];              // -2 unused, -1 open segment, >= 0 row that ended

    const int t = xcd_tile(blockIdx.x, ntiles);
    if (t < 0) return;
    const int tid = threadIdx.x, lane = tid & (WAVE - 1);
    // BS == 1: tell the compiler that the wave index is uniform (scalar loop control).  With blocks the
    // generated code measured 3 % slower that way, so there it stays a per-lane value.
    const int wave = BS == 1 ? __builtin_amdgcn_readfirstlane(tid / WAVE) : tid / WAVE;
    const int t0 = t * T;
    const int cnt = (nnz - t0 < T) ? nnz - t0 : T;
    const int t1 = t0 + cnt;
    const int col = blockIdx.y * KW + lane * VEC;
    const bool active = col < k;
    const int lcol = active ? col : 0;            // lanes past the last column load column 0 and store nothing

    for (int i = tid; i < T; i += THREADS) sflag[i] = -1;
    if (tid < 2 * NW) srec_row[tid] = -2;

    const int r0 = tile_row[t], r1 = tile_row[t + 1];
    const bool has_carry = (t > 0) && (pos[r0] < t0);
    const int rbeg = (t == 0) ? 0 : r0;
    const bool straddle = pos[r1] != t1;          // row r1 continues into the next tile
    const int rend = straddle ? r1 + 1 : r1;
    if (tid == 0 && blockIdx.y == 0 && !has_carry) carry_row[t] = -1;
    __syncthreads();

    // ---- row ends of this tile, zero rows
    for (int rb = rbeg + wave * WAVE; rb < rend; rb += THREADS) {
        const int r = rb + lane;
        const bool valid = r < rend;
        const int ps = valid ? pos[r] : 0, pe = valid ? pos[r + 1] : 1;
        if (valid && pe > ps) {
            const int e = pe - 1 - t0;
            if (e >= 0 && e < cnt) sflag[e] = r;
        }
        unsigned long long empty = __ballot(valid && pe == ps);
        while (empty) {
            const int j = __ffsll((long long)empty) - 1;
            empty &= empty - 1;
            if (active) {
                const float z[VEC] = {};
#pragma unroll
                for (int ii = 0; ii < BS; ++ii) st_vec<VEC>(C + ((long long)(rb + j) * BS + ii) * ldc + col, z);
            }
        }
    }
    __syncthreads();

    // ---- the wave's positions
    const int CH = T / NW;
    const int wbeg = wave * CH < cnt ? wave * CH : cnt;
    const int wend = wbeg + CH < cnt ? wbeg + CH : cnt;
    float acc[BS][VEC] = {};
    bool seen = false;

    auto flush = [&](int f) {
        if (!seen) {
            seen = true;
#pragma unroll
            for (int ii = 0; ii < BS; ++ii)
#pragma unroll
                for (int v = 0; v < VEC; ++v) srec[2 * wave][ii][lane * VEC + v] = acc[ii][v];
            if (lane == 0) srec_row[2 * wave] = f;
        } else if (active) {
#pragma unroll
            for (int ii = 0; ii < BS; ++ii) st_vec<VEC>(C + ((long long)f * BS + ii) * ldc + col, acc[ii]);
        }
#pragma unroll
        for (int ii = 0; ii < BS; ++ii)
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[ii][v] = 0.0f;
    };

    // crd and vals of 64 positions, one per lane; requested one batch ahead of their use
    int c_n = 0;
    float v_n[BS * BS];
    auto fetch = [&](int base) {
        c_n = 0;
#pragma unroll
        for (int e = 0; e < BS * BS; ++e) v_n[e] = 0.0f;
        if (base + lane < wend) {
            const int p = t0 + base + lane;
            c_n = ld_stream(crd + p);
            if constexpr (BS == 1) v_n[0] = ld_stream(vals + p);
            else {
#pragma unroll
                for (int q = 0; q < BS * BS / 4; ++q) {
                    const v4f v = *reinterpret_cast<const v4f *>(vals + (long long)p * (BS * BS) + q * 4);
                    v_n[4 * q + 0] = v.x; v_n[4 * q + 1] = v.y; v_n[4 * q + 2] = v.z; v_n[4 * q + 3] = v.w;
                }
            }
        }
    };
    constexpr bool AHEAD = BS == 1;               // blocks: 16 more registers per lane would cost occupancy
    if (AHEAD) fetch(wbeg);
    for (int base = wbeg; base < wend; base += WAVE) {
        const int n = wend - base < WAVE ? wend - base : WAVE;
        if (!AHEAD) fetch(base);
        const int c_l = c_n;
        const int f_l = lane < n ? sflag[base + lane] : -1;
        float v_l[BS * BS];
#pragma unroll
        for (int e = 0; e < BS * BS; ++e) v_l[e] = v_n[e];
        if (AHEAD) fetch(base + WAVE);
        for (int j0 = 0; j0 < n; j0 += U) {
            float b[U][BS][VEC];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int j = (j0 + u) & (WAVE - 1);       // lanes past n hold column 0, value 0
                const long long c = rl(c_l, j);
#pragma unroll
                for (int ji = 0; ji < BS; ++ji) {
                    if (BS == 1 || active) ld_vec<VEC>(b[u][ji], B + (c * BS + ji) * ldb + lcol);
                    else {
#pragma unroll
                        for (int v = 0; v < VEC; ++v) b[u][ji][v] = 0.0f;
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int j = j0 + u;
                if (j < n) {
#pragma unroll
                    for (int ii = 0; ii < BS; ++ii)
#pragma unroll
                        for (int ji = 0; ji < BS; ++ji) {
                            const float a = rl(v_l[ii * BS + ji], j);
#pragma unroll
                            for (int v = 0; v < VEC; ++v) acc[ii][v] = fmaf(a, b[u][ji][v], acc[ii][v]);
                        }
                    const int f = rl(f_l, j);
                    if (f >= 0) flush(f);
                }
            }
        }
    }
    if (wbeg < wend) {
        const int slot = seen ? 2 * wave + 1 : 2 * wave;
#pragma unroll
        for (int ii = 0; ii < BS; ++ii)
#pragma unroll
            for (int v = 0; v < VEC; ++v) srec[slot][ii][lane * VEC + v] = acc[ii][v];
        if (lane == 0) srec_row[slot] = -1;
    }
    __syncthreads();

    // ---- chain the records (wave 0)
    if (wave != 0) return;
    float run[BS][VEC] = {};
    const long long wcarry = (long long)BS * k;
    auto finalize = [&](int r) {
        if (has_carry && r == r0) {
            if (active) {
#pragma unroll
                for (int ii = 0; ii < BS; ++ii)
#pragma unroll
                    for (int v = 0; v < VEC; ++v) carry_val[(long long)t * wcarry + (long long)ii * k + col + v] = run[ii][v];
            }
            if (lane == 0 && blockIdx.y == 0) carry_row[t] = r;
        } else if (active) {
#pragma unroll
            for (int ii = 0; ii < BS; ++ii) st_vec<VEC>(C + ((long long)r * BS + ii) * ldc + col, run[ii]);
        }
#pragma unroll
        for (int ii = 0; ii < BS; ++ii)
#pragma unroll
            for (int v = 0; v < VEC; ++v) run[ii][v] = 0.0f;
    };
    for (int rec = 0; rec < 2 * NW; ++rec) {
        const int code = srec_row[rec];
        if (code == -2) continue;
#pragma unroll
        for (int ii = 0; ii < BS; ++ii)
#pragma unroll
            for (int v = 0; v < VEC; ++v) run[ii][v] += srec[rec][ii][lane * VEC + v];
        if (code >= 0) finalize(code);
    }
    if (straddle) finalize(r1);
}

bool spmm_csr_tile_ok(int32_t tile) { return tile == 256 || tile == 512 || tile == 1024 || tile == 2048; }
bool bcsr_tile_ok(int32_t tile) { return tile == 64 || tile == 128 || tile == 256 || tile == 512; }

// Widest per-lane vector the operands allow, not wider than needed to cover k with one chunk.
static int pick_vec(const float *B, int32_t k, int64_t ldb, const float *C, int64_t ldc)
{
    const uintptr_t a = reinterpret_cast<uintptr_t>(B) | reinterpret_cast<uintptr_t>(C);
    int vec = 1;
    if (k > 64 && k % 2 == 0 && ldb % 2 == 0 && ldc % 2 == 0 && (a & 7) == 0) vec = 2;
    if (k > 128 && k % 4 == 0 && ldb % 4 == 0 && ldc % 4 == 0 && (a & 15) == 0) vec = 4;
    return vec;
}

template <int BS>
static hipError_t launch_spmm_pos(int32_t rows, int32_t nnz, const int32_t *pos, const int32_t *crd,
                                  const float *vals, const float *B, int32_t k, int64_t ldb, float *C,
                                  int64_t ldc, int32_t tile, const Workspace &w, hipStream_t s)
{
    const int ntiles = (int)(((int64_t)nnz + tile - 1) / tile);
    if (ntiles == 0) return hipSuccess;
    int vec = pick_vec(B, k, ldb, C, ldc);
    if (BS == 8 && vec == 4) vec = 2;             // 8 x 8 blocks: the LDS records of four columns per lane do not fit
    const int kw = WAVE * vec;
    const dim3 grid(xcd_grid(ntiles), (k + kw - 1) / kw);
    const size_t lds = (size_t)tile * sizeof(int);
#define PSK_GO(V)                                                                                              \
    PSK_LAUNCH((k_spmm_pos<BS, V>), grid, dim3(256), lds, s, rows, nnz, pos, crd, vals, B, k,          \
                       (long long)ldb, C, (long long)ldc, w.tile_row, w.carry_row, w.carry_val, ntiles, tile)
    if (vec == 4) {
        if constexpr (BS < 8) PSK_GO(4);
    } else if (vec == 2) PSK_GO(2);
    else PSK_GO(1);
#undef PSK_GO
    return take_launch_status();
}

hipError_t launch_spmm_csr_main(int32_t rows, int32_t nnz, const int32_t *pos, const int32_t *crd,
                                const float *vals, const float *B, int32_t k, int64_t ldb, float *C,
                                int64_t ldc, int32_t tile, const Workspace &w, hipStream_t s)
{
    if (k <= 32) return launch_spmm_csr_narrow(rows, nnz, pos, crd, vals, B, k, ldb, C, ldc, tile, w, s);
    return launch_spmm_pos<1>(rows, nnz, pos, crd, vals, B, k, ldb, C, ldc, tile, w, s);
}

hipError_t launch_spmm_bcsr_main(int32_t bs, int32_t brows, int32_t nblocks, const int32_t *pos, const int32_t *crd,
                                 const float *vals, const float *B, int32_t k, int64_t ldb, float *C,
                                 int64_t ldc, int32_t tile, const Workspace &w, hipStream_t s)
{
    if (bs == 2) return launch_spmm_pos<2>(brows, nblocks, pos, crd, vals, B, k, ldb, C, ldc, tile, w, s);
    if (bs == 4) return launch_spmm_pos<4>(brows, nblocks, pos, crd, vals, B, k, ldb, C, ldc, tile, w, s);
    if (bs == 8) return launch_spmm_pos<8>(brows, nblocks, pos, crd, vals, B, k, ldb, C, ldc, tile, w, s);
    return hipErrorInvalidValue;
}

// Row-split SpMM baseline: one wave per row, lanes over columns (64 at a time), serial over the
// row's positions.
__global__ __launch_bounds__(256) void k_spmm_wave_per_row(int rows, const int *__restrict__ pos,
                                                           const int *__restrict__ crd,
                                                           const float *__restrict__ vals,
                                                           const float *__restrict__ B, int k, long long ldb,
                                                           float *__restrict__ C, long long ldc)
{
    const int lane = threadIdx.x & (WAVE - 1);
    const int r = blockIdx.x * (256 / WAVE) + threadIdx.x / WAVE;
    if (r >= rows) return;
    const int ps = pos[r], pe = pos[r + 1];
    for (int c0 = 0; c0 < k; c0 += WAVE) {
        const int col = c0 + lane;
        float acc = 0.0f;
        if (col < k)
            for (int p = ps; p < pe; ++p) acc = fmaf(vals[p], B[(long long)crd[p] * ldb + col], acc);
        if (col < k) C[(long long)r * ldc + col] = acc;
    }
}

hipError_t launch_spmm_rowsplit(int32_t rows, const int32_t *pos, const int32_t *crd, const float *vals,
                                const float *B, int32_t k, int64_t ldb, float *C, int64_t ldc, hipStream_t s)
{
    if (rows == 0) return hipSuccess;
    PSK_LAUNCH(k_spmm_wave_per_row, dim3((rows + 3) / 4), dim3(256), 0, s, rows, pos, crd, vals, B, k,
                       (long long)ldb, C, (long long)ldc);
    return take_launch_status();
}

}  // namespace psk
