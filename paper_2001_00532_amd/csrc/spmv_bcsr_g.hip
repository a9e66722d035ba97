// BCSR SpMV for 2x2 and 8x8 dense blocks (4x4 has its own kernel).  Same position cut at the block
// level, same row logic and carry records; only the mapping of lanes to the dense inner levels of the
// hierarchy (Section 1) differs with the block edge BS:
//   BS = 2: one lane per block: one 16-byte load holds the block, one 8-byte gather its two x values,
//           the lane forms both row sums;
//   BS = 8: sixteen lanes per block: lane q loads four values of block row q/2 (columns 4*(q%2)..),
//           gathers the matching 16 bytes of x, forms a 4-term dot product and adds its neighbour's.
#include "psk_dev.h"
#include "psk_internal.h"

namespace psk {

template <int BS, int TB>
__global__ __launch_bounds__(256) void k_spmv_bcsr_g(int brows, int nblocks, const int *__restrict__ pos,
                                                     const int *__restrict__ crd,
                                                     const float *__restrict__ vals,
                                                     const float *__restrict__ x, float *__restrict__ y,
                                                     const int *__restrict__ tile_row,
                                                     int *__restrict__ carry_row,
                                                     float *__restrict__ carry_val, int ntiles)
{
    static_assert(BS == 2 || BS == 8, "block edge");
    constexpr int THREADS = 256, NW = THREADS / WAVE;
    constexpr int LPB = BS * BS / 4;               // lanes per block
    constexpr int BPP = THREADS / LPB;             // blocks per pass of the workgroup
    constexpr int NPASS = TB / BPP;
    constexpr int RPI = THREADS / BS;              // block rows per iteration of the row loop
    constexpr int LONG = BS == 2 ? 48 : 16;        // blocks of one block row in the tile from which a wave takes over
    constexpr int MAXLONG = TB / LONG > 0 ? TB / LONG : 1;
    static_assert(TB % BPP == 0 && NPASS >= 1, "tile must be a multiple of the blocks per pass");
    __shared__ float sprod[TB * BS];               // [block][row in block]
    __shared__ int slong[MAXLONG * 3];
    __shared__ int nlong;

    const int t = xcd_tile(blockIdx.x, ntiles);
    if (t < 0) return;
    const int tid = threadIdx.x, lane = tid & (WAVE - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / WAVE);
    const int q = tid % LPB, bl = tid / LPB;
    const int t0 = t * TB;
    const int cnt = (nblocks - t0 < TB) ? nblocks - t0 : TB;
    const int t1 = t0 + cnt;

    const int r0 = tile_row[t], r1 = tile_row[t + 1];

    v4f a[NPASS];
    int jb[NPASS];
#pragma unroll
    for (int g = 0; g < NPASS; ++g) {
        const int i = g * BPP + bl;
        a[g] = v4f{0.f, 0.f, 0.f, 0.f};
        jb[g] = 0;
        if (i < cnt) {
            const long long p = t0 + i;
            a[g] = ld_stream(reinterpret_cast<const v4f *>(vals + p * (BS * BS) + q * 4));
            jb[g] = ld_stream(crd + p);
        }
    }
    const int p_r0 = pos[r0], p_r1 = pos[r1];

    if (tid == 0) nlong = 0;
#pragma unroll
    for (int g = 0; g < NPASS; ++g) {
        const int i = g * BPP + bl;
        if constexpr (BS == 2) {
            float s0 = 0.0f, s1 = 0.0f;
            if (i < cnt) {
                const v2f b = *reinterpret_cast<const v2f *>(x + (long long)jb[g] * 2);
                s0 = a[g].x * b.x + a[g].y * b.y;
                s1 = a[g].z * b.x + a[g].w * b.y;
            }
            sprod[i * 2] = s0;
            sprod[i * 2 + 1] = s1;
        } else {
            float d = 0.0f;
            if (i < cnt) {
                const v4f b = *reinterpret_cast<const v4f *>(x + (long long)jb[g] * 8 + (q & 1) * 4);
                d = a[g].x * b.x + a[g].y * b.y + a[g].z * b.z + a[g].w * b.w;
            }
            d += dpp_mov<0xB1>(d);                 // the other half of the same block row (lane ^ 1)
            if ((q & 1) == 0) sprod[i * 8 + (q >> 1)] = d;
        }
    }

    const bool has_carry = (t > 0) && (p_r0 < t0);
    const int rbeg = (t == 0) ? 0 : r0;
    const int rend = (p_r1 == t1) ? r1 : r1 + 1;
    if (tid == 0 && !has_carry) carry_row[t] = -1;
    __syncthreads();

    const int ii = tid % BS, rl = tid / BS;
    auto emit = [&](int r, int e, float s) {
        if (has_carry && r == r0) { carry_row[t] = r; carry_val[(long long)t * BS + e] = s; }
        else y[(long long)r * BS + e] = s;
    };
    for (int rb = rbeg; rb < rend; rb += RPI) {
        const int r = rb + rl;
        if (r < rend) {
            int lo = pos[r] - t0, hi = pos[r + 1] - t0;
            lo = lo < 0 ? 0 : lo;
            hi = hi > cnt ? cnt : hi;
            if (hi - lo < LONG) {
                float s = 0.0f;
                for (int i = lo; i < hi; ++i) s += sprod[i * BS + ii];
                emit(r, ii, s);
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
        for (int i = lo + lane / BS; i < hi; i += WAVE / BS) s += sprod[i * BS + lane % BS];
#pragma unroll
        for (int m = BS; m < WAVE; m <<= 1) s += __shfl_xor(s, m, WAVE);
        if (lane < BS) emit(r, lane, s);
    }
}

bool bcsr_g_tile_ok(int32_t bs, int32_t tile)
{
    if (bs == 2) return tile == 512 || tile == 1024 || tile == 2048;
    if (bs == 8) return tile == 32 || tile == 64 || tile == 128;
    return false;
}

hipError_t launch_spmv_bcsr_g_main(int32_t bs, int32_t brows, int32_t nblocks, const int32_t *pos, const int32_t *crd,
                                   const float *vals, const float *x, float *y, int32_t tile, const Workspace &w,
                                   hipStream_t s)
{
    const int ntiles = (int)(((int64_t)nblocks + tile - 1) / tile);
    if (ntiles == 0) return hipSuccess;
    const int grid = xcd_grid(ntiles);
#define PSK_GO(B, TB)                                                                                              \
    PSK_LAUNCH((k_spmv_bcsr_g<B, TB>), dim3(grid), dim3(256), 0, s, brows, nblocks, pos, crd, vals, x, y, \
                       w.tile_row, w.carry_row, w.carry_val, ntiles)
    if (bs == 2) {
        switch (tile) {
            case 512: PSK_GO(2, 512); break;
            case 1024: PSK_GO(2, 1024); break;
            case 2048: PSK_GO(2, 2048); break;
            default: return hipErrorInvalidValue;
        }
    } else if (bs == 8) {
        switch (tile) {
            case 32: PSK_GO(8, 32); break;
            case 64: PSK_GO(8, 64); break;
            case 128: PSK_GO(8, 128); break;
            default: return hipErrorInvalidValue;
        }
    } else {
        return hipErrorInvalidValue;
    }
#undef PSK_GO
    return take_launch_status();
}

}  // namespace psk
