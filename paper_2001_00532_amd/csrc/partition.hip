// Position cut and the carry fix-up: the two small kernels every operation shares.
#include "psk_dev.h"
#include "psk_internal.h"

namespace psk {

// tile_row[t] = largest i in [0, rows] with pos[i] <= min(t*tile, nnz)   (Section 6.2: the first
// coordinate of a tile of the position space is recovered by a binary search over pos).
// One lane per table entry; pos[0] = 0 makes i = 0 always admissible.
__global__ __launch_bounds__(256) void k_partition(int rows, int nnz, const int *__restrict__ pos,
                                                   int tile, int ntiles, int *__restrict__ tile_row,
                                                   int *__restrict__ gap)
{
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t == 0 && gap) { gap[0] = 0; gap[1] = 0; }
    if (t > ntiles) return;
    const long long first = (long long)t * tile;
    const int target = first < nnz ? (int)first : nnz;
    int lo = 0, hi = rows;
    while (lo < hi) {
        const int mid = lo + ((hi - lo + 1) >> 1);
        if (pos[mid] <= target) lo = mid; else hi = mid - 1;
    }
    tile_row[t] = lo;
}

// The same table from one pass over the rows instead of one search per tile (Section 5, "Divide",
// names both ways of locating a tile's start: an O(log n) search or an O(n) walk).  Row r owns the
// first position of every tile t with pos[r] <= t*tile < pos[r+1]; each non-empty row writes those
// entries.  Every tile start lies in exactly one non-empty row, so the table is filled exactly once.
// No dependent loads: the kernel streams pos at memory speed, which beats the search's chain of
// log2(rows) cache misses as long as pos itself is not huge.  Rows that own many tile starts are
// written by their whole wave.
__global__ __launch_bounds__(256) void k_partition_scan(int rows, int nnz, const int *__restrict__ pos, int tile,
                                                        int shift, int ntiles, int *__restrict__ tile_row,
                                                        int vec_ok, int *__restrict__ gap)
{
    constexpr int RPT = 4;                                   // rows per thread
    const int g = blockIdx.x * blockDim.x + threadIdx.x;
    const int lane = threadIdx.x & (WAVE - 1);
    const int rbase = g * RPT;
    if (g == 0) {
        tile_row[ntiles] = rows;
        if (gap) { gap[0] = 0; gap[1] = 0; }
    }
    int p[RPT + 1];
    if (vec_ok && rbase + RPT <= rows) {
        const v4i v = *reinterpret_cast<const v4i *>(pos + rbase);
        p[0] = v.x; p[1] = v.y; p[2] = v.z; p[3] = v.w;
        p[4] = pos[rbase + RPT];
    } else {
#pragma unroll
        for (int i = 0; i <= RPT; ++i) p[i] = rbase + i <= rows ? pos[rbase + i] : nnz;
    }
#pragma unroll
    for (int i = 0; i < RPT; ++i) {
        const int r = rbase + i;
        int t_lo = 0, t_hi = -1;
        if (r < rows && p[i + 1] > p[i]) {
            if (shift >= 0) {
                t_lo = (int)(((long long)p[i] + tile - 1) >> shift);
                t_hi = (p[i + 1] - 1) >> shift;
            } else {
                t_lo = (int)(((long long)p[i] + tile - 1) / tile);
                t_hi = (p[i + 1] - 1) / tile;
            }
        }
        const int n = t_hi - t_lo + 1;                       // tile starts inside this row
        if (n > 0 && n <= 16)
            for (int t = t_lo; t <= t_hi; ++t) tile_row[t] = r;
        unsigned long long big = __ballot(n > 16);
        while (big) {
            const int src = __ffsll((long long)big) - 1;
            big &= big - 1;
            const int lo = __shfl(t_lo, src, WAVE), hi = __shfl(t_hi, src, WAVE), row = __shfl(r, src, WAVE);
            for (int t = lo + lane; t <= hi; t += WAVE) tile_row[t] = row;
        }
    }
}

// method: 0 = choose, 1 = binary search per tile, 2 = one scan over the rows
hipError_t launch_partition(int64_t rows, int64_t nnz, const int32_t *pos, int32_t tile, int method,
                            int32_t *tile_row, hipStream_t s, int32_t *gap)
{
    const int64_t ntiles = nnz <= 0 ? 0 : (nnz + tile - 1) / tile;
    if (method == 0) method = (ntiles > 0 && rows <= (int64_t(1) << 23)) ? 2 : 1;
    if (method == 2 && ntiles > 0) {
        int shift = -1;
        if ((tile & (tile - 1)) == 0) { shift = 0; while ((1 << shift) < tile) ++shift; }
        const int vec_ok = (reinterpret_cast<uintptr_t>(pos) & 15) == 0;
        const int64_t threads = (rows + 3) / 4;
        PSK_LAUNCH(k_partition_scan, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, (int)rows,
                           (int)nnz, pos, tile, shift, (int)ntiles, tile_row, vec_ok, gap);
        return take_launch_status();
    }
    const int64_t n = ntiles + 1;
    PSK_LAUNCH(k_partition, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, (int)rows, (int)nnz, pos,
                       tile, (int)ntiles, tile_row, gap);
    return take_launch_status();
}

// Gather-locality probe: of up to 16384 evenly spaced positions p, how many have their successor's
// column within the same 128-byte line of x (0 <= crd[p+1] - crd[p] < 32)?  One workgroup; result[0] =
// hits, result[1] = samples.
__global__ __launch_bounds__(1024) void k_probe_locality(int nnz, const int *__restrict__ crd, int *__restrict__ result)
{
    __shared__ int swave[1024 / WAVE];
    const int samples = nnz - 1 < 16384 ? nnz - 1 : 16384;
    const long long stride = samples > 0 ? (long long)(nnz - 1) / samples : 1;
    int hits = 0;
    for (int i = threadIdx.x; i < samples; i += 1024) {
        const long long p = i * stride;
        const int d = crd[p + 1] - crd[p];
        hits += (d >= 0 && d < 32) ? 1 : 0;
    }
#pragma unroll
    for (int m = 1; m < WAVE; m <<= 1) hits += __shfl_xor(hits, m, WAVE);
    if ((threadIdx.x & (WAVE - 1)) == 0) swave[threadIdx.x / WAVE] = hits;
    __syncthreads();
    if (threadIdx.x == 0) {
        int tot = 0;
        for (int w = 0; w < 1024 / WAVE; ++w) tot += swave[w];
        result[0] = tot;
        result[1] = samples;
    }
}

hipError_t launch_probe_locality(int32_t nnz, const int32_t *crd, int32_t *result, hipStream_t s)
{
    PSK_LAUNCH(k_probe_locality, dim3(1), dim3(1024), 0, s, nnz, crd, result);
    return take_launch_status();
}

// Longest row: result[0] = max_i (pos[i+1] - pos[i]); result must hold 0 before the launch.
__global__ __launch_bounds__(256) void k_max_row(int rows, const int *__restrict__ pos, int *__restrict__ result)
{
    int m = 0;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < rows; i += (long long)gridDim.x * blockDim.x) {
        const int len = pos[i + 1] - pos[i];
        m = len > m ? len : m;
    }
#pragma unroll
    for (int k = 1; k < WAVE; k <<= 1) {
        const int o = __shfl_xor(m, k, WAVE);
        m = o > m ? o : m;
    }
    if ((threadIdx.x & (WAVE - 1)) == 0 && m > 0) atomicMax(result, m);
}

hipError_t launch_max_row(int32_t rows, const int32_t *pos, int32_t *result, hipStream_t s)
{
    hipError_t e = launch_fill_zero(reinterpret_cast<float *>(result), 1, s);   // +0.0f is the integer 0
    if (e != hipSuccess || rows <= 0) return e;
    int64_t blocks = ((int64_t)rows + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    PSK_LAUNCH(k_max_row, dim3((unsigned)blocks), dim3(256), 0, s, rows, pos, result);
    return take_launch_status();
}

// Structural check of a CSR index structure.  result[c] counts the violations of condition c:
// 1: pos[0] != 0;  2: pos[i+1] < pos[i];  3: pos[rows] != nnz;  4: crd[p] outside [0, cols).
// result[0..4] must hold 0 before the launch.
__global__ __launch_bounds__(256) void k_validate_csr(int rows, int cols, int nnz, const int *__restrict__ pos,
                                                      const int *__restrict__ crd, int *__restrict__ result)
{
    const long long g = (long long)blockIdx.x * blockDim.x + threadIdx.x, stride = (long long)gridDim.x * blockDim.x;
    int bad2 = 0, bad4 = 0;
    for (long long i = g; i < rows; i += stride) bad2 += pos[i + 1] < pos[i] ? 1 : 0;
    for (long long p = g; p < nnz; p += stride) {
        const int c = crd[p];
        bad4 += (c < 0 || c >= cols) ? 1 : 0;
    }
    if (g == 0) {
        if (pos[0] != 0) atomicAdd(result + 1, 1);
        if (pos[rows] != nnz) atomicAdd(result + 3, 1);
    }
    if (bad2) atomicAdd(result + 2, bad2);
    if (bad4) atomicAdd(result + 4, bad4);
}

hipError_t launch_validate_csr(int32_t rows, int32_t cols, int32_t nnz, const int32_t *pos, const int32_t *crd,
                               int32_t *result, hipStream_t s)
{
    hipError_t e = launch_fill_zero(reinterpret_cast<float *>(result), 8, s);
    if (e != hipSuccess) return e;
    int64_t work = rows > nnz ? rows : nnz;
    int64_t blocks = (work + 255) / 256;
    blocks = blocks < 1 ? 1 : (blocks > 4096 ? 4096 : blocks);
    PSK_LAUNCH(k_validate_csr, dim3((unsigned)blocks), dim3(256), 0, s, rows, cols, nnz, pos, crd, result);
    return take_launch_status();
}

__global__ __launch_bounds__(256) void k_fill_zero(float *__restrict__ p, long long n)
{
    long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long stride = (long long)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = 0.0f;
}

hipError_t launch_fill_zero(float *p, int64_t n, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    PSK_LAUNCH(k_fill_zero, dim3((unsigned)blocks), dim3(256), 0, s, p, (long long)n);
    return take_launch_status();
}

__global__ __launch_bounds__(256) void k_fill_zero_2d(float *__restrict__ p, long long rows, int width, long long ld)
{
    const long long n = rows * width;
    long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long stride = (long long)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[(i / width) * ld + i % width] = 0.0f;
}

// rows x width block of a row-major array with leading dimension ld
hipError_t launch_fill_zero_2d(float *p, int64_t rows, int32_t width, int64_t ld, hipStream_t s)
{
    if (ld == width) return launch_fill_zero(p, rows * width, s);
    if (rows <= 0 || width <= 0) return hipSuccess;
    int64_t blocks = (rows * width + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    PSK_LAUNCH(k_fill_zero_2d, dim3((unsigned)blocks), dim3(256), 0, s, p, (long long)rows, width, (long long)ld);
    return take_launch_status();
}

// Carry fix-up.  Tile t left carry_row[t] = r >= 0 when its first positions belong to a row r that
// began in an earlier tile, together with `width` partial sums.  The records of one row sit in
// consecutive tiles: from the tile after the one holding pos[r] to the tile holding the row's last
// position, so the lane that sees the head of a run knows its length from pos[r+1] alone and no load
// in the walk depends on another.  The run is added in tile order, in fp64, to the owner's partial
// result.  out element (r, e) lives at out[(r*nsub + e / k) * ld + e % k].
__device__ __forceinline__ int run_length(const int *__restrict__ pos, const int *__restrict__ pos2, int r, int t,
                                          int tile, int shift, int ntiles)
{
    const int last = (pos2 ? pos2[pos[r + 1]] : pos[r + 1]) - 1;
    int e = shift >= 0 ? last >> shift : last / tile;
    int len = e - t + 1;
    len = len < 1 ? 1 : len;
    return len > ntiles - t ? ntiles - t : len;
}

// width = 1 (SpMV): a lane per tile; runs of more than 8 records are summed by the whole wave.
// V = float: fp32 records and output, summed in fp64.  V = double: all fp64.
// Workgroups from `carry_groups` on (launched only for the CSR SpMV) clear the runs of empty rows that tiles listed in
// `gap` instead of walking them (gap[0] = number of runs, then first and end row of each): every row r of a run with
// pos[r] = pos[r+1] becomes 0; rows with entries were written by their tiles.  The last of these workgroups to finish
// resets the two counters, so that a product which reuses the table (no partition step) starts from an empty list.
template <typename V>
__global__ __launch_bounds__(256) void k_carry_fixup1(int ntiles, long long ld, int tile, int shift,
                                                      const int *__restrict__ pos,
                                                      const int *__restrict__ carry_row,
                                                      const V *__restrict__ carry_val,
                                                      V *__restrict__ out, int carry_groups, int *__restrict__ gap)
{
    if ((int)blockIdx.x >= carry_groups) {
        const int fillers = (int)gridDim.x - carry_groups, me = (int)blockIdx.x - carry_groups;
        int n = gap[0];
        if (n == 0) return;                      // the usual case: no run was listed, nothing to clear or to reset
        n = n < ntiles ? n : ntiles;
        for (int e = 0; e < n; ++e) {
            const long long lo = gap[2 + 2 * e], hi = gap[3 + 2 * e];
            for (long long r = lo + (long long)me * 256 + threadIdx.x; r < hi; r += (long long)fillers * 256)
                if (pos[r] == pos[r + 1]) out[r * ld] = V(0);
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            __threadfence();
            if (atomicAdd(&gap[1], 1) == fillers - 1) { gap[0] = 0; gap[1] = 0; }
        }
        return;
    }
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    const int lane = threadIdx.x & (WAVE - 1);
    int r = -1, len = 0;
    if (t < ntiles) {
        r = carry_row[t];
        const int prev = t > 0 ? carry_row[t - 1] : -1;
        if (r >= 0 && prev != r) len = run_length(pos, nullptr, r, t, tile, shift, ntiles);
    }
    if (len > 0 && len <= 8) {
        V v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = i < len ? carry_val[t + i] : V(0);
        double sum = 0.0;
#pragma unroll
        for (int i = 0; i < 8; ++i) sum += (double)v[i];
        out[r * ld] = (V)((double)out[r * ld] + sum);
    }
    unsigned long long big = __ballot(len > 8);
    while (big) {
        const int src = __ffsll((long long)big) - 1;
        big &= big - 1;
        const int t0 = __shfl(t, src, WAVE), n = __shfl(len, src, WAVE), row = __shfl(r, src, WAVE);
        double acc = 0.0;
        for (int u = lane; u < n; u += WAVE) acc += (double)carry_val[t0 + u];
#pragma unroll
        for (int m = 1; m < WAVE; m <<= 1) acc += __shfl_xor(acc, m, WAVE);
        if (lane == src) out[row * ld] = (V)((double)out[row * ld] + acc);
    }
}

// any width: a lane per (tile, element); the run is walked eight records at a time.
__global__ __launch_bounds__(256) void k_carry_fixup(int ntiles, int width, int nsub, int k, long long ld, int tile,
                                                     int shift, const int *__restrict__ pos,
                                                     const int *__restrict__ pos2,
                                                     const int *__restrict__ rowmap,
                                                     const int *__restrict__ carry_row,
                                                     const float *__restrict__ carry_val,
                                                     float *__restrict__ out)
{
    const long long g = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long total = (long long)ntiles * width;
    if (g >= total) return;
    int t, e;
    if (total <= 0xffffffffll) {          // the usual case: a 32-bit division is several times cheaper
        const unsigned gg = (unsigned)g;
        t = (int)(gg / (unsigned)width);
        e = (int)(gg - (unsigned)t * (unsigned)width);
    } else {
        t = (int)(g / width);
        e = (int)(g % width);
    }
    const int r = carry_row[t];
    if (r < 0) return;
    if (t > 0 && carry_row[t - 1] == r) return;
    const int len = run_length(pos, pos2, r, t, tile, shift, ntiles);
    double sum = 0.0;
    for (int u = 0; u < len; u += 8) {
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = u + i < len ? carry_val[(long long)(t + u + i) * width + e] : 0.0f;
#pragma unroll
        for (int i = 0; i < 8; ++i) sum += (double)v[i];
    }
    const long long row = rowmap ? rowmap[r] : r;
    float *dst = out + (row * nsub + e / k) * ld + e % k;
    *dst = (float)((double)*dst + sum);
}

hipError_t launch_carry_fixup(int32_t ntiles, int32_t nsub, int32_t k, int64_t ld, int32_t tile, const int32_t *pos,
                              const Workspace &w, float *out, hipStream_t s, const int32_t *pos2,
                              const int32_t *rowmap, bool gaps)
{
    const int width = nsub * k;
    gaps = gaps && width == 1 && !pos2 && !rowmap && ntiles >= 1;
    if (ntiles <= 1 && !gaps) return hipSuccess;   // tile 0 never has a carry
    int shift = -1;
    if ((tile & (tile - 1)) == 0) { shift = 0; while ((1 << shift) < tile) ++shift; }
    if (width == 1 && !pos2 && !rowmap) {
        const int carry_groups = ntiles <= 1 ? 0 : (ntiles + 255) / 256;
        int *gap = gaps ? w.gap : nullptr;
        PSK_LAUNCH(k_carry_fixup1<float>, dim3((unsigned)(carry_groups + (gaps ? kGapFillGroups : 0))), dim3(256), 0, s,
                   ntiles, (long long)ld, tile, shift, pos, w.carry_row, w.carry_val, out, carry_groups, gap);
        return take_launch_status();
    }
    const int64_t n = (int64_t)ntiles * width;
    PSK_LAUNCH(k_carry_fixup, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, ntiles, width, nsub, k,
                       (long long)ld, tile, shift, pos, pos2, rowmap, w.carry_row, w.carry_val, out);
    return take_launch_status();
}

hipError_t launch_carry_fixup_f64(int32_t ntiles, int32_t tile, const int32_t *pos, const Workspace &w, double *out,
                                  hipStream_t s, bool gaps)
{
    gaps = gaps && ntiles >= 1;
    if (ntiles <= 1 && !gaps) return hipSuccess;
    int shift = -1;
    if ((tile & (tile - 1)) == 0) { shift = 0; while ((1 << shift) < tile) ++shift; }
    const int carry_groups = ntiles <= 1 ? 0 : (ntiles + 255) / 256;
    int *gap = gaps ? w.gap : nullptr;
    PSK_LAUNCH(k_carry_fixup1<double>, dim3((unsigned)(carry_groups + (gaps ? kGapFillGroups : 0))), dim3(256), 0, s, ntiles,
               1ll, tile, shift, pos, w.carry_row, reinterpret_cast<const double *>(w.carry_val), out, carry_groups, gap);
    return take_launch_status();
}

}  // namespace psk
