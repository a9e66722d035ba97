// BCSR (4x4 dense blocks) SpMV in position space.  The position cut is taken at the block level
// (Section 3: a cut may be placed at any level of the coordinate hierarchy); the two dense inner
// levels of the hierarchy (Section 1) become straight-line code: four lanes share a block, each
// does one block row as a 16-byte load and a 4-term dot product with a 16-byte gather of x.
#include "psk_dev.h"
#include "psk_internal.h"

namespace psk {

// Sum over the 16 lanes of a wave that share (lane % 4); every such lane receives the result.
__device__ __forceinline__ float wave_sum_mod4(float v)
{
    v += __shfl_xor(v, 4, WAVE);
    v += __shfl_xor(v, 8, WAVE);
    v += __shfl_xor(v, 16, WAVE);
    v += __shfl_xor(v, 32, WAVE);
    return v;
}

// One workgroup of 256 threads per tile of TB blocks; thread (blk = tid/4, ii = tid%4) handles row ii
// of blocks blk, blk+64, ...  Same row logic as the CSR kernel with block rows in place of rows and
// four partial sums (one per ii) per block row.
template <int TB>
__global__ __launch_bounds__(256) void k_spmv_bcsr4(int brows, int nblocks, const int *__restrict__ pos,
                                                    const int *__restrict__ crd,
                                                    const float *__restrict__ vals,
                                                    const float *__restrict__ x, float *__restrict__ y,
                                                    const int *__restrict__ tile_row,
                                                    int *__restrict__ carry_row,
                                                    float *__restrict__ carry_val, int ntiles)
{
    constexpr int THREADS = 256, NW = THREADS / WAVE, NPASS = TB / 64;
    constexpr int LONG = 16;                 // blocks of one block row inside the tile handled by a whole wave
    constexpr int MAXLONG = TB / LONG;
    __shared__ float sprod[skewed_size<4>(TB * 4)];
    __shared__ int slong[MAXLONG * 3];
    __shared__ int nlong;
    __shared__ float swave[NW][4];

    const int t = xcd_tile(blockIdx.x, ntiles);
    if (t < 0) return;
    const int tid = threadIdx.x, lane = tid & (WAVE - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / WAVE);   // tells the compiler it is uniform
    const int ii = tid & 3;
    const int t0 = t * TB;
    const int cnt = (nblocks - t0 < TB) ? nblocks - t0 : TB;
    const int t1 = t0 + cnt;

    // the dependent chain tile_row -> pos is started first and runs underneath the streaming loads
    const int r0 = tile_row[t], r1 = tile_row[t + 1];

    v4f a[NPASS];
    int jb[NPASS];
#pragma unroll
    for (int g = 0; g < NPASS; ++g) {
        const int i = g * 64 + (tid >> 2);
        a[g] = v4f{0.f, 0.f, 0.f, 0.f};
        jb[g] = 0;
        if (i < cnt) {
            const long long p = t0 + i;
            a[g] = ld_stream(reinterpret_cast<const v4f *>(vals + p * 16 + ii * 4));
            jb[g] = ld_stream(crd + p);
        }
    }

    const int p_r0 = pos[r0], p_r1 = pos[r1];
    const int rbeg = (t == 0) ? 0 : r0;
    int my_lo = 0, my_hi = 0;                     // pos pair of the first block row this lane looks at
    if (rbeg + (tid >> 2) < brows) {
        my_lo = pos[rbeg + (tid >> 2)];
        my_hi = pos[rbeg + (tid >> 2) + 1];
    }

    float prod[NPASS];
#pragma unroll
    for (int g = 0; g < NPASS; ++g) {
        const int i = g * 64 + (tid >> 2);
        prod[g] = 0.0f;
        if (i < cnt) {
            const v4f b = *reinterpret_cast<const v4f *>(x + (long long)jb[g] * 4);
            prod[g] = a[g].x * b.x + a[g].y * b.y + a[g].z * b.z + a[g].w * b.w;
        }
    }

    const bool has_carry = (t > 0) && (p_r0 < t0);
    const int rend = (p_r1 == t1) ? r1 : r1 + 1;
    if (tid == 0 && !has_carry) carry_row[t] = -1;

    if (rend - rbeg == 1) {   // the tile lies inside one block row
        float s = 0.0f;
#pragma unroll
        for (int g = 0; g < NPASS; ++g) s += prod[g];
        s = wave_sum_mod4(s);
        if (lane < 4) swave[wave][lane] = s;
        __syncthreads();
        if (tid < 4) {
            float tot = swave[0][tid];
#pragma unroll
            for (int w = 1; w < NW; ++w) tot += swave[w][tid];
            if (has_carry) { carry_row[t] = rbeg; carry_val[(long long)t * 4 + tid] = tot; }
            else y[(long long)rbeg * 4 + tid] = tot;
        }
        return;
    }

    if (tid == 0) nlong = 0;
#pragma unroll
    for (int g = 0; g < NPASS; ++g) sprod[skew<4>(g * 256 + tid)] = prod[g];   // index = block*4 + ii
    __syncthreads();
    for (int rb = rbeg; rb < rend; rb += THREADS / 4) {
        const int r = rb + (tid >> 2);
        if (r < rend) {
            int lo = my_lo - t0, hi = my_hi - t0;
            if (r + THREADS / 4 < rend) { my_lo = pos[r + THREADS / 4]; my_hi = pos[r + THREADS / 4 + 1]; }
            lo = lo < 0 ? 0 : lo;
            hi = hi > cnt ? cnt : hi;
            if (hi - lo < LONG) {
                float s = 0.0f;
                for (int i = lo; i < hi; ++i) s += sprod[skew<4>(i * 4 + ii)];
                if (has_carry && r == r0) { carry_row[t] = r; carry_val[(long long)t * 4 + ii] = s; }
                else y[(long long)r * 4 + ii] = s;
            } else if (ii == 0) {
                const int e = atomicAdd(&nlong, 1);
                if (e < MAXLONG) { slong[3 * e] = r; slong[3 * e + 1] = lo; slong[3 * e + 2] = hi; }
            }
        }
    }
    __syncthreads();
    const int nl = nlong < MAXLONG ? nlong : MAXLONG;
    for (int e = wave; e < nl; e += NW) {
        const int r = slong[3 * e], lo = slong[3 * e + 1], hi = slong[3 * e + 2];
        float s = 0.0f;
        for (int i = lo + (lane >> 2); i < hi; i += WAVE / 4) s += sprod[skew<4>(i * 4 + (lane & 3))];
        s = wave_sum_mod4(s);
        if (lane < 4) {
            if (has_carry && r == r0) { carry_row[t] = r; carry_val[(long long)t * 4 + lane] = s; }
            else y[(long long)r * 4 + lane] = s;
        }
    }
}

hipError_t launch_spmv_bcsr4_main(int32_t brows, int32_t nblocks, const int32_t *pos, const int32_t *crd,
                                  const float *vals, const float *x, float *y, int32_t tile,
                                  const Workspace &w, hipStream_t s)
{
    const int ntiles = (int)(((int64_t)nblocks + tile - 1) / tile);
    if (ntiles == 0) return hipSuccess;
    const int grid = xcd_grid(ntiles);
#define PSK_GO(TB)                                                                                           \
    PSK_LAUNCH((k_spmv_bcsr4<TB>), dim3(grid), dim3(256), 0, s, brows, nblocks, pos, crd, vals, x, y, \
                       w.tile_row, w.carry_row, w.carry_val, ntiles)
    switch (tile) {
        case 64: PSK_GO(64); break;
        case 128: PSK_GO(128); break;
        case 256: PSK_GO(256); break;
        case 512: PSK_GO(512); break;
        default: return hipErrorInvalidValue;
    }
#undef PSK_GO
    return take_launch_status();
}

}  // namespace psk
