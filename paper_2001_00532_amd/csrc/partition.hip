// Position cut and the carry fix-up: the two small kernels every operation shares.
#include "psk_dev.h"
#include "psk_internal.h"

namespace psk {

// tile_row[t] = largest i in [0, rows] with pos[i] <= min(t*tile, nnz)   (Section 6.2: the first
// coordinate of a tile of the position space is recovered by a binary search over pos).
// One lane per table entry; pos[0] = 0 makes i = 0 always admissible.
__global__ __launch_bounds__(256) void k_partition(int rows, int nnz, const int *__restrict__ pos,
                                                   int tile, int ntiles, int *__restrict__ tile_row)
{
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
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

hipError_t launch_partition(int64_t rows, int64_t nnz, const int32_t *pos, int32_t tile, int32_t *tile_row,
                            hipStream_t s)
{
    const int64_t ntiles = nnz <= 0 ? 0 : (nnz + tile - 1) / tile;
    const int64_t n = ntiles + 1;
    hipLaunchKernelGGL(k_partition, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, (int)rows, (int)nnz, pos,
                       tile, (int)ntiles, tile_row);
    return hipGetLastError();
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
    hipLaunchKernelGGL(k_fill_zero, dim3((unsigned)blocks), dim3(256), 0, s, p, (long long)n);
    return hipGetLastError();
}

// Carry fix-up.  Tile t left carry_row[t] = r >= 0 when its first positions belong to a row r that
// began in an earlier tile, together with `width` partial sums.  Carry rows are non-decreasing in t
// and the tiles of one row are consecutive, so the records of a row form a run; the lane that sees
// the head of a run adds the whole run, in tile order and in fp64, to the owner's partial result.
// out element (r, e) lives at out[(r*nsub + e / k) * ld + e % k].
__global__ __launch_bounds__(256) void k_carry_fixup(int ntiles, int width, int nsub, int k, long long ld,
                                                     const int *__restrict__ carry_row,
                                                     const float *__restrict__ carry_val,
                                                     float *__restrict__ out)
{
    const long long g = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= (long long)ntiles * width) return;
    const int t = (int)(g / width), e = (int)(g % width);
    const int r = carry_row[t];
    if (r < 0) return;
    if (t > 0 && carry_row[t - 1] == r) return;
    double sum = 0.0;
    for (int u = t; u < ntiles && carry_row[u] == r; ++u) sum += (double)carry_val[(long long)u * width + e];
    float *dst = out + ((long long)r * nsub + e / k) * ld + e % k;
    *dst = (float)((double)*dst + sum);
}

hipError_t launch_carry_fixup(int32_t ntiles, int32_t nsub, int32_t k, int64_t ld, const Workspace &w,
                              float *out, hipStream_t s)
{
    if (ntiles <= 1) return hipSuccess;   // tile 0 never has a carry
    const int width = nsub * k;
    const int64_t n = (int64_t)ntiles * width;
    hipLaunchKernelGGL(k_carry_fixup, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, ntiles, width, nsub, k,
                       (long long)ld, w.carry_row, w.carry_val, out);
    return hipGetLastError();
}

}  // namespace psk
