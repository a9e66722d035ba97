// CSR SpMV: position-space kernel (appendix "SPMV on a GPU", Sections 3/5/6) and the two
// coordinate-space baselines of Section 8.3.
#include "psk_dev.h"
#include "psk_internal.h"

namespace psk {

// One workgroup per tile of T = THREADS*NPT consecutive positions of A.
//
//  1. stream: every thread loads NPT (crd, vals) pairs with coalesced loads, gathers x and keeps the
//     products in registers (the schedule's per-thread temporary + unrolled load loop).
//  2. rows of the tile: tile_row[t] .. tile_row[t+1] bound the rows that own positions of this tile
//     (the coordinate recovery of Section 6.2, done once per tile by k_partition).  The tile WRITES
//     y for the rows that begin inside it (plus the empty rows at its end and, for tile 0, the empty
//     rows before the first position); the part of a row that began in an earlier tile goes to this
//     tile's carry record instead of an atomic add.
//  3. reduction:  - the whole tile lies in one row: registers -> wave butterfly -> LDS across waves;
//                 - otherwise products go to LDS, one thread sums each short row segment serially,
//                   segments of >= LONG positions are queued and summed by a whole wave each.
//     Every row segment has a fixed summation order, so results are deterministic.
//
// VEC: 16-byte loads (needs 16-byte aligned crd/vals); otherwise 4-byte loads, lane-consecutive.
template <int THREADS, int NPT, bool VEC>
__global__ __launch_bounds__(THREADS) void k_spmv_pos(int rows, int nnz, const int *__restrict__ pos,
                                                      const int *__restrict__ crd,
                                                      const float *__restrict__ vals,
                                                      const float *__restrict__ x, float *__restrict__ y,
                                                      const int *__restrict__ tile_row,
                                                      int *__restrict__ carry_row,
                                                      float *__restrict__ carry_val, int ntiles)
{
    constexpr int T = THREADS * NPT;
    constexpr int NW = THREADS / WAVE;
    constexpr int LONG = 32;
    constexpr int MAXLONG = T / LONG;
    static_assert(NPT % 4 == 0, "NPT must be a multiple of 4");
    __shared__ float sprod[skewed_size<1>(T)];
    __shared__ int slong[MAXLONG * 3];
    __shared__ int nlong;
    __shared__ float swave[NW];

    const int t = xcd_tile(blockIdx.x, ntiles);
    if (t < 0) return;
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid / WAVE;
    const int t0 = t * T;
    const int cnt = (nnz - t0 < T) ? nnz - t0 : T;
    const int t1 = t0 + cnt;

    // ---- 1. stream + gather + multiply
    float prod[NPT];
    if (cnt == T) {
        if (VEC) {
            v4i c[NPT / 4];
            v4f v[NPT / 4];
#pragma unroll
            for (int g = 0; g < NPT / 4; ++g) {
                const int off = t0 + (g * THREADS + tid) * 4;
                c[g] = ld_stream(reinterpret_cast<const v4i *>(crd + off));
                v[g] = ld_stream(reinterpret_cast<const v4f *>(vals + off));
            }
#pragma unroll
            for (int g = 0; g < NPT / 4; ++g) {
                prod[4 * g + 0] = v[g].x * x[c[g].x];
                prod[4 * g + 1] = v[g].y * x[c[g].y];
                prod[4 * g + 2] = v[g].z * x[c[g].z];
                prod[4 * g + 3] = v[g].w * x[c[g].w];
            }
        } else {
            int c[NPT];
            float v[NPT];
#pragma unroll
            for (int g = 0; g < NPT; ++g) {
                c[g] = ld_stream(crd + t0 + g * THREADS + tid);
                v[g] = ld_stream(vals + t0 + g * THREADS + tid);
            }
#pragma unroll
            for (int g = 0; g < NPT; ++g) prod[g] = v[g] * x[c[g]];
        }
    } else {   // last tile: guarded
#pragma unroll
        for (int g = 0; g < NPT; ++g) {
            const int i = VEC ? ((g / 4) * THREADS + tid) * 4 + (g & 3) : g * THREADS + tid;
            prod[g] = (i < cnt) ? vals[t0 + i] * x[crd[t0 + i]] : 0.0f;
        }
    }

    // ---- 2. rows of this tile
    const int r0 = tile_row[t], r1 = tile_row[t + 1];
    const bool has_carry = (t > 0) && (pos[r0] < t0);
    const int rbeg = (t == 0) ? 0 : r0;
    const int rend = (pos[r1] == t1) ? r1 : r1 + 1;   // last tile: r1 = rows and pos[rows] = nnz = t1
    if (tid == 0 && !has_carry) carry_row[t] = -1;

    // ---- 3a. the tile lies inside a single row
    if (rend - rbeg == 1) {
        float s = 0.0f;
#pragma unroll
        for (int g = 0; g < NPT; ++g) s += prod[g];
        s = wave_sum(s);
        if (lane == 0) swave[wave] = s;
        __syncthreads();
        if (tid == 0) {
            float tot = swave[0];
#pragma unroll
            for (int w = 1; w < NW; ++w) tot += swave[w];
            if (has_carry) { carry_row[t] = rbeg; carry_val[t] = tot; }
            else y[rbeg] = tot;
        }
        return;
    }

    // ---- 3b. several rows: products to LDS in position order
    if (tid == 0) nlong = 0;
#pragma unroll
    for (int g = 0; g < NPT; ++g) {
        const int i = VEC ? ((g / 4) * THREADS + tid) * 4 + (g & 3) : g * THREADS + tid;
        sprod[skew<1>(i)] = prod[g];
    }
    __syncthreads();
    for (int r = rbeg + tid; r < rend; r += THREADS) {
        int lo = pos[r] - t0, hi = pos[r + 1] - t0;
        lo = lo < 0 ? 0 : lo;
        hi = hi > cnt ? cnt : hi;
        if (hi - lo < LONG) {
            float s = 0.0f;
            for (int i = lo; i < hi; ++i) s += sprod[skew<1>(i)];
            if (has_carry && r == r0) { carry_row[t] = r; carry_val[t] = s; }
            else y[r] = s;
        } else {
            const int e = atomicAdd(&nlong, 1);
            if (e < MAXLONG) { slong[3 * e] = r; slong[3 * e + 1] = lo; slong[3 * e + 2] = hi; }
        }
    }
    __syncthreads();
    const int nl = nlong < MAXLONG ? nlong : MAXLONG;
    for (int e = wave; e < nl; e += NW) {
        const int r = slong[3 * e], lo = slong[3 * e + 1], hi = slong[3 * e + 2];
        float s = 0.0f;
        for (int i = lo + lane; i < hi; i += WAVE) s += sprod[skew<1>(i)];
        s = wave_sum(s);
        if (lane == 0) {
            if (has_carry && r == r0) { carry_row[t] = r; carry_val[t] = s; }
            else y[r] = s;
        }
    }
}

bool spmv_csr_tile_ok(int32_t tile)
{
    return tile == 256 || tile == 512 || tile == 1024 || tile == 2048 || tile == 4096;
}

template <int THREADS, int NPT>
static void launch_pos(bool vec, int grid, hipStream_t s, int rows, int nnz, const int *pos, const int *crd,
                       const float *vals, const float *x, float *y, const Workspace &w, int ntiles)
{
    if (vec)
        hipLaunchKernelGGL((k_spmv_pos<THREADS, NPT, true>), dim3(grid), dim3(THREADS), 0, s, rows, nnz, pos, crd,
                           vals, x, y, w.tile_row, w.carry_row, w.carry_val, ntiles);
    else
        hipLaunchKernelGGL((k_spmv_pos<THREADS, NPT, false>), dim3(grid), dim3(THREADS), 0, s, rows, nnz, pos, crd,
                           vals, x, y, w.tile_row, w.carry_row, w.carry_val, ntiles);
}

hipError_t launch_spmv_csr_main(int32_t rows, int32_t nnz, const int32_t *pos, const int32_t *crd,
                                const float *vals, const float *x, float *y, int32_t tile,
                                const Workspace &w, hipStream_t s)
{
    const int ntiles = (int)(((int64_t)nnz + tile - 1) / tile);
    if (ntiles == 0) return hipSuccess;
    const int grid = xcd_grid(ntiles);
    const bool vec = ((reinterpret_cast<uintptr_t>(crd) | reinterpret_cast<uintptr_t>(vals)) & 15) == 0;
    switch (tile) {
        case 256:  launch_pos<64, 4>(vec, grid, s, rows, nnz, pos, crd, vals, x, y, w, ntiles); break;
        case 512:  launch_pos<128, 4>(vec, grid, s, rows, nnz, pos, crd, vals, x, y, w, ntiles); break;
        case 1024: launch_pos<256, 4>(vec, grid, s, rows, nnz, pos, crd, vals, x, y, w, ntiles); break;
        case 2048: launch_pos<256, 8>(vec, grid, s, rows, nnz, pos, crd, vals, x, y, w, ntiles); break;
        case 4096: launch_pos<256, 16>(vec, grid, s, rows, nnz, pos, crd, vals, x, y, w, ntiles); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------ coordinate-space baselines

// Thread per row (appendix "SpMV Thread per Row on GPU"): rows split over workgroups, one row per
// thread, serial sum.  Uncoalesced and divergent by construction -- it is the baseline of Section 8.3.
__global__ __launch_bounds__(256) void k_spmv_thread_per_row(int rows, const int *__restrict__ pos,
                                                             const int *__restrict__ crd,
                                                             const float *__restrict__ vals,
                                                             const float *__restrict__ x,
                                                             float *__restrict__ y)
{
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= rows) return;
    float s = 0.0f;
    for (int p = pos[r]; p < pos[r + 1]; ++p) s += vals[p] * x[crd[p]];
    y[r] = s;
}

// Wave per row (appendix "SpMV Warp per Row on GPU"): the lanes of a wave stride over the positions
// of one row, then reduce with the wave butterfly.
__global__ __launch_bounds__(256) void k_spmv_wave_per_row(int rows, const int *__restrict__ pos,
                                                           const int *__restrict__ crd,
                                                           const float *__restrict__ vals,
                                                           const float *__restrict__ x,
                                                           float *__restrict__ y)
{
    const int lane = threadIdx.x & (WAVE - 1);
    const int r = blockIdx.x * (256 / WAVE) + threadIdx.x / WAVE;
    if (r >= rows) return;
    const int pe = pos[r + 1];
    float s = 0.0f;
    for (int p = pos[r] + lane; p < pe; p += WAVE) s += vals[p] * x[crd[p]];
    s = wave_sum(s);
    if (lane == 0) y[r] = s;
}

hipError_t launch_spmv_rowsplit(int32_t rows, const int32_t *pos, const int32_t *crd, const float *vals,
                                const float *x, float *y, int variant, hipStream_t s)
{
    if (rows == 0) return hipSuccess;
    if (variant == 0)
        hipLaunchKernelGGL(k_spmv_thread_per_row, dim3((rows + 255) / 256), dim3(256), 0, s, rows, pos, crd, vals, x,
                           y);
    else
        hipLaunchKernelGGL(k_spmv_wave_per_row, dim3((rows + 3) / 4), dim3(256), 0, s, rows, pos, crd, vals, x, y);
    return hipGetLastError();
}

}  // namespace psk
