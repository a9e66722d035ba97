// MTTKRP on a three-level compressed tensor in position space (appendix "MTTKRP on a GPU"):
//     A(i,j) = B(i,k,l) * C(k,j) * D(l,j)
// Schedule: the k and l loops are fused, then i with them; the fused loop runs over the positions of
// B's leaf level, split into tiles (workgroups) and wave chunks; j is split over the lanes; the loop
// over a wave's positions is innermost.  Section 3: a position loop keeps track of every coordinate
// above the cut the same way it tracks the row of a CSR matrix -- here two levels, fiber and slice.
#include "psk_dev.h"
#include "psk_internal.h"

namespace psk {

// tile_fiber[t] = largest q in [0, nfibers] with pos_l[q] <= min(t*tile, nnz); tile_slice[t] = largest s in
// [0, nslices] with pos_k[s] <= tile_fiber[t]: two chained binary searches (Section 6.2), one lane per entry.
__global__ __launch_bounds__(256) void k_partition_csf3(int nslices, int nfibers, int nnz,
                                                        const int *__restrict__ pos_k,
                                                        const int *__restrict__ pos_l, int tile, int ntiles,
                                                        int *__restrict__ tile_slice,
                                                        int *__restrict__ tile_fiber)
{
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t > ntiles) return;
    const long long first = (long long)t * tile;
    const int target = first < nnz ? (int)first : nnz;
    int lo = 0, hi = nfibers;
    while (lo < hi) {
        const int mid = lo + ((hi - lo + 1) >> 1);
        if (pos_l[mid] <= target) lo = mid; else hi = mid - 1;
    }
    const int q = lo;
    lo = 0; hi = nslices;
    while (lo < hi) {
        const int mid = lo + ((hi - lo + 1) >> 1);
        if (pos_k[mid] <= q) lo = mid; else hi = mid - 1;
    }
    tile_fiber[t] = q;
    tile_slice[t] = lo;
}

hipError_t launch_partition_csf3(int32_t nslices, int32_t nfibers, int32_t nnz, const int32_t *pos_k,
                                 const int32_t *pos_l, int32_t tile, int32_t *tile_slice, int32_t *tile_fiber,
                                 hipStream_t s)
{
    const int ntiles = nnz <= 0 ? 0 : (int)(((int64_t)nnz + tile - 1) / tile);
    PSK_LAUNCH(k_partition_csf3, dim3((ntiles + 1 + 255) / 256), dim3(256), 0, s, nslices, nfibers, nnz, pos_k,
                       pos_l, tile, ntiles, tile_slice, tile_fiber);
    return take_launch_status();
}

// One workgroup (4 waves) per tile of T leaf positions and per chunk of 64*VEC columns.
//
// Tile metadata in LDS: sflag[i] = s if leaf position i is the last leaf of slice s (slices play the role
// the rows play in SpMM; a slice's leaves are pos_l[pos_k[s]] .. pos_l[pos_k[s+1]]), and sk[i] = the mode-k
// coordinate k of the fiber that owns leaf i, stored as ~k on the fiber's last leaf in the tile (filled fiber
// by fiber from the tile's window of pos_l; fibers with >= LONGF leaves in the tile are filled by a whole
// wave).  Slices without leaves that fall into the
// tile's write range get zero rows.
// A wave walks its leaves 64 at a time: l, k, flag and value are loaded one per lane and broadcast with
// v_readlane, so that the rows D[l,:] and C[k,:] are wave-uniform, contiguous loads; U rows of D are
// requested before the first multiply.  Within a fiber the product is regrouped by distributivity,
// A(i,:) += C(k,:) * sum_l B(i,k,l) D(l,:), so the C row is requested once, where the fiber's partial sum
// closes (its last leaf in the tile, or the wave's last leaf), not once per leaf: a cache hit between every
// two misses of the D gather costs bandwidth, because the vector memory pipeline returns in order.
// Segments, records, carries: as in the SpMM kernel (the first and last open segments of each wave are
// chained by wave 0; a chain whose slice began before the tile becomes the tile's carry record).
// G > 1 (narrow factor matrices, j <= 64/G, VEC = 1): the wave is split into G groups of 64/G lanes and in one
// step the groups take G consecutive leaves, so that one load instruction fetches G rows of D.  A lane keeps
// its group's share of the open fiber and of the open slice; a fiber end multiplies every share by the C row
// (no exchange needed: the product distributes over the shares), a slice end adds the shares across groups.
template <int VEC, int G>
__global__ __launch_bounds__(256) void k_mttkrp_pos(int nslices, int nnz, const int *__restrict__ crd_i,
                                                    const int *__restrict__ pos_k,
                                                    const int *__restrict__ crd_k,
                                                    const int *__restrict__ pos_l,
                                                    const int *__restrict__ crd_l,
                                                    const float *__restrict__ vals,
                                                    const float *__restrict__ C, long long ldc,
                                                    const float *__restrict__ D, long long ldd, int jdim,
                                                    float *__restrict__ A, long long lda,
                                                    const int *__restrict__ tile_slice,
                                                    const int *__restrict__ tile_fiber,
                                                    int *__restrict__ carry_row,
                                                    float *__restrict__ carry_val, int ntiles, int T)
{
    static_assert(G == 1 || VEC == 1, "lane groups only with one column per lane");
    constexpr int THREADS = 256, NW = THREADS / WAVE, GW = WAVE / G, KW = GW * VEC, LONGF = 32;
    constexpr int U = G > 1 ? 4 : (VEC == 4 ? 4 : 8);   // steps whose D rows are in flight together
    extern __shared__ int smeta[];                // sflag[T], sk[T], long-fiber queue [3 * T / LONGF]
    int *sflag = smeta, *sk = smeta + T, *slong = smeta + 2 * T;
    __shared__ float srec[2 * NW][KW];
    __shared__ int srec_row[2 * NW];              // -2 unused, -1 open segment, >= 0 slice that ended
    __shared__ int nlong;

    const int t = xcd_tile(blockIdx.x, ntiles);
    if (t < 0) return;
    const int tid = threadIdx.x, lane = tid & (WAVE - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / WAVE);   // tells the compiler it is uniform
    const int t0 = t * T;
    const int cnt = (nnz - t0 < T) ? nnz - t0 : T;
    const int t1 = t0 + cnt;
    const int g = lane / GW, gl = lane % GW;      // group of the lane, lane inside the group (G = 1: 0, lane)
    const int col = blockIdx.y * KW + gl * VEC;
    const bool active = col < jdim;
    const bool writer = active && g == 0;         // group 0 stores on behalf of the wave
    const int lcol = active ? col : 0;            // lanes past the last column load column 0 and store nothing

    for (int i = tid; i < T; i += THREADS) { sflag[i] = -1; sk[i] = 0; }
    if (tid < 2 * NW) srec_row[tid] = -2;
    if (tid == 0) nlong = 0;

    const int r0 = tile_slice[t], r1 = tile_slice[t + 1];
    const int q0 = tile_fiber[t], q1 = tile_fiber[t + 1];
    const int leaf_r0 = pos_l[pos_k[r0]], leaf_r1 = pos_l[pos_k[r1]];   // first leaf of slices r0, r1
    const bool has_carry = (t > 0) && (leaf_r0 < t0);
    const int rbeg = (t == 0) ? 0 : r0;
    const bool straddle = leaf_r1 != t1;          // slice r1 continues into the next tile
    const int rend = straddle ? r1 + 1 : r1;
    const int qend = (pos_l[q1] != t1) ? q1 + 1 : q1;   // fibers with leaves in this tile: q0 .. qend-1
    if (tid == 0 && blockIdx.y == 0 && !has_carry) carry_row[t] = -1;
    __syncthreads();

    // ---- slice ends of this tile, zero rows for slices without leaves
    for (int rb = rbeg + wave * WAVE; rb < rend; rb += THREADS) {
        const int r = rb + lane;
        const bool valid = r < rend;
        const int ps = valid ? pos_l[pos_k[r]] : 0, pe = valid ? pos_l[pos_k[r + 1]] : 1;
        if (valid && pe > ps) {
            const int e = pe - 1 - t0;
            if (e >= 0 && e < cnt) sflag[e] = r;
        }
        unsigned long long empty = __ballot(valid && pe == ps);
        while (empty) {
            const int j = __ffsll((long long)empty) - 1;
            empty &= empty - 1;
            if (writer) {
                const float z[VEC] = {};
                const long long row = crd_i ? crd_i[rb + j] : rb + j;
                st_vec<VEC>(A + row * lda + col, z);
            }
        }
    }
    // ---- mode-k coordinate of every leaf of the tile
    for (int q = q0 + tid; q < qend; q += THREADS) {
        int lo = pos_l[q] - t0, hi = pos_l[q + 1] - t0;
        lo = lo < 0 ? 0 : lo;
        hi = hi > cnt ? cnt : hi;
        const int kk = crd_k[q];
        if (hi - lo < LONGF) {
            for (int i = lo; i < hi; ++i) sk[i] = (i == hi - 1) ? ~kk : kk;
        } else {
            const int e = atomicAdd(&nlong, 1);
            if (e < T / LONGF) { slong[3 * e] = kk; slong[3 * e + 1] = lo; slong[3 * e + 2] = hi; }
        }
    }
    __syncthreads();
    {
        const int nl = nlong < T / LONGF ? nlong : T / LONGF;
        for (int e = wave; e < nl; e += NW) {
            const int kk = slong[3 * e], lo = slong[3 * e + 1], hi = slong[3 * e + 2];
            for (int i = lo + lane; i < hi; i += WAVE) sk[i] = (i == hi - 1) ? ~kk : kk;
        }
    }
    __syncthreads();

    // ---- the wave's leaves
    const int CH = T / NW;
    const int wbeg = wave * CH < cnt ? wave * CH : cnt;
    const int wend = wbeg + CH < cnt ? wbeg + CH : cnt;
    float acc[VEC] = {};
    float facc[VEC] = {};                         // sum of b * D(l, :) over the leaves of the open fiber
    bool seen = false;

    auto group_sum = [&](float v) {               // sum over the G lanes that hold the same column
#pragma unroll
        for (int m = GW; m < WAVE; m <<= 1) v += __shfl_xor(v, m, WAVE);
        return v;
    };
    auto flush = [&](int f) {                     // G > 1: acc already holds the sum over the groups
        if (!seen) {
            seen = true;
            if (g == 0) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) srec[2 * wave][gl * VEC + v] = acc[v];
            }
            if (lane == 0) srec_row[2 * wave] = f;
        } else if (writer) {
            const long long row = crd_i ? crd_i[f] : f;
            st_vec<VEC>(A + row * lda + col, acc);
        }
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[v] = 0.0f;
    };

    // crd_l and vals of 64 leaves, one per lane; requested one batch ahead of their use
    int l_n = 0;
    float v_n = 0.0f;
    auto fetch = [&](int base) {
        l_n = 0;
        v_n = 0.0f;
        if (base + lane < wend) {
            l_n = ld_stream(crd_l + t0 + base + lane);
            v_n = ld_stream(vals + t0 + base + lane);
        }
    };
    fetch(wbeg);
    for (int base = wbeg; base < wend; base += WAVE) {
        const int n = wend - base < WAVE ? wend - base : WAVE;
        const int l_l = l_n;
        const float v_l = v_n;
        int k_l = lane < n ? sk[base + lane] : 0;
        const int f_l = lane < n ? sflag[base + lane] : -1;
        fetch(base + WAVE);
        if (base + lane == wend - 1 && k_l >= 0) k_l = ~k_l;   // the wave's last leaf closes its fiber's partial sum
        if constexpr (G > 1) {
        for (int j0 = 0; j0 < n; j0 += U * G) {
            float c[U], d[U], a[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int jj = (j0 + u * G + g) & (WAVE - 1);      // this group's leaf in step u
                const long long ll = __shfl(l_l, jj, WAVE);        // lanes past n hold coordinate 0, value 0, no flag
                const int ke = __shfl(k_l, jj, WAVE);
                a[u] = __shfl(v_l, jj, WAVE);
                c[u] = 0.0f;
                if (ke < 0) c[u] = C[(long long)(~ke) * ldc + lcol];   // this group's leaf closes a fiber
                d[u] = D[ll * ldd + lcol];
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int s0 = j0 + u * G;                          // first leaf of the step
                if (s0 < n) {
                    const float term = (s0 + g < n) ? a[u] * d[u] : 0.0f;
                    bool added = false;
#pragma unroll
                    for (int e = 0; e < G; ++e) {
                        if (rl(k_l, (s0 + e) & (WAVE - 1)) < 0) {   // leaf s0 + e is the last of its fiber
                            if (!added && g <= e) { facc[0] += term; added = true; }
                            const float ce = __shfl(c[u], e * GW + gl, WAVE);   // the C row group e fetched
                            acc[0] = fmaf(ce, facc[0], acc[0]);
                            facc[0] = 0.0f;
                            const int f = rl(f_l, (s0 + e) & (WAVE - 1));
                            if (f >= 0) {                           // ... and of its slice
                                acc[0] = group_sum(acc[0]);
                                flush(f);
                            }
                        }
                    }
                    if (!added) facc[0] += term;
                }
            }
        }
        } else {
        for (int j0 = 0; j0 < n; j0 += U) {
            float c[U][VEC], d[U][VEC];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int j = (j0 + u) & (WAVE - 1);       // lanes past n hold coordinate 0, value 0, no flag
                const int ke = rl(k_l, j);
                const long long ll = rl(l_l, j);
                // The C row is needed once per fiber, where its partial sum closes (uniform over the wave).
                if (ke < 0) {
                    ld_vec<VEC>(c[u], C + (long long)(~ke) * ldc + lcol);
                } else {
#pragma unroll
                    for (int v = 0; v < VEC; ++v) c[u][v] = 0.0f;
                }
                ld_vec<VEC>(d[u], D + ll * ldd + lcol);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int j = j0 + u;
                if (j < n) {
                    const float a = rl(v_l, j);
#pragma unroll
                    for (int v = 0; v < VEC; ++v) facc[v] = fmaf(a, d[u][v], facc[v]);
                    if (rl(k_l, j) < 0) {
#pragma unroll
                        for (int v = 0; v < VEC; ++v) { acc[v] = fmaf(c[u][v], facc[v], acc[v]); facc[v] = 0.0f; }
                        const int f = rl(f_l, j);
                        if (f >= 0) flush(f);
                    }
                }
            }
        }
        }
    }
    if (wbeg < wend) {
        const int slot = seen ? 2 * wave + 1 : 2 * wave;
        if constexpr (G > 1) acc[0] = group_sum(acc[0]);
        if (g == 0) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) srec[slot][gl * VEC + v] = acc[v];
        }
        if (lane == 0) srec_row[slot] = -1;
    }
    __syncthreads();

    // ---- chain the records (wave 0, group 0)
    if (wave != 0 || g != 0) return;
    float run[VEC] = {};
    auto finalize = [&](int r) {
        if (has_carry && r == r0) {
            if (active) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) carry_val[(long long)t * jdim + col + v] = run[v];
            }
            if (lane == 0 && blockIdx.y == 0) carry_row[t] = r;
        } else if (active) {
            const long long row = crd_i ? crd_i[r] : r;
            st_vec<VEC>(A + row * lda + col, run);
        }
#pragma unroll
        for (int v = 0; v < VEC; ++v) run[v] = 0.0f;
    };
    for (int rec = 0; rec < 2 * NW; ++rec) {
        const int code = srec_row[rec];
        if (code == -2) continue;
#pragma unroll
        for (int v = 0; v < VEC; ++v) run[v] += srec[rec][gl * VEC + v];
        if (code >= 0) finalize(code);
    }
    if (straddle) finalize(r1);
}

bool mttkrp_tile_ok(int32_t tile) { return tile == 256 || tile == 512 || tile == 1024 || tile == 2048; }

hipError_t launch_mttkrp_main(int32_t nslices, int32_t nnz, const int32_t *crd_i, const int32_t *pos_k,
                              const int32_t *crd_k, const int32_t *pos_l, const int32_t *crd_l, const float *vals,
                              const float *C, int64_t ldc, const float *D, int64_t ldd, int32_t j, float *A,
                              int64_t lda, int32_t tile, const Workspace &w, const int32_t *tile_fiber,
                              hipStream_t s)
{
    const int ntiles = (int)(((int64_t)nnz + tile - 1) / tile);
    if (ntiles == 0) return hipSuccess;
    const uintptr_t al = reinterpret_cast<uintptr_t>(C) | reinterpret_cast<uintptr_t>(D) | reinterpret_cast<uintptr_t>(A);
    int vec = 1;
    if (j > 64 && j % 2 == 0 && ldc % 2 == 0 && ldd % 2 == 0 && lda % 2 == 0 && (al & 7) == 0) vec = 2;
    if (j > 128 && j % 4 == 0 && ldc % 4 == 0 && ldd % 4 == 0 && lda % 4 == 0 && (al & 15) == 0) vec = 4;
    const int groups = j <= 8 ? 8 : (j <= 16 ? 4 : (j <= 32 ? 2 : 1));
    const int kw = WAVE * vec / groups;
    const dim3 grid(xcd_grid(ntiles), (j + kw - 1) / kw);
    const size_t lds = ((size_t)2 * tile + 3 * (size_t)(tile / 32)) * sizeof(int);
#define PSK_GO(V, GG)                                                                                           \
    PSK_LAUNCH((k_mttkrp_pos<V, GG>), grid, dim3(256), lds, s, nslices, nnz, crd_i, pos_k, crd_k, pos_l,    \
                       crd_l, vals, C, (long long)ldc, D, (long long)ldd, j, A, (long long)lda, w.tile_row,         \
                       tile_fiber, w.carry_row, w.carry_val, ntiles, tile)
    if (groups == 8) PSK_GO(1, 8);
    else if (groups == 4) PSK_GO(1, 4);
    else if (groups == 2) PSK_GO(1, 2);
    else if (vec == 4) PSK_GO(4, 1);
    else if (vec == 2) PSK_GO(2, 1);
    else PSK_GO(1, 1);
#undef PSK_GO
    return take_launch_status();
}

}  // namespace psk
