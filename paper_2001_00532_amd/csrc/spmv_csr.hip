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
// MODE 0: 4-byte loads, lane-consecutive positions (works for any alignment).
// MODE 1: 16-byte loads (crd and vals 16-byte aligned), each lane keeps four consecutive positions.
template <int MODE, int THREADS>
__device__ __forceinline__ int tile_index(int g, int tid)
{
    if (MODE == 0) return g * THREADS + tid;
    return ((g / 4) * THREADS + tid) * 4 + (g & 3);
}

// VARIANT 0: one pass, carries.  1: a column pass (window [clo, chi), accum adds to earlier passes).
// 2: one pass with the schedule's atomics instead of carries (baseline).
// 4: one pass over a DCSR operand: `rows` counts the stored rows, row s of the hierarchy is row rowmap[s]
//    of y (Section 3: the cut may be taken at any level of any coordinate hierarchy; y is zero-filled
//    by the caller because rows that are not stored are written by nobody).
// 5: a column pass (as 1) over a DCSR operand (as 4).
// 3: one pass without the per-thread temporary and without the unrolled load loop (the ablation of
//    Section 8.3): each thread walks its positions in a rolled loop, one load -> gather -> multiply -> LDS
//    store after the other.
// 7: the whole matrix is one tile (nnz <= T): no table, no carries, no fix-up -- one launch per product for
//    problems of a few thousand entries, which are bound by launch latency.
// 6: one pass with unit values: vals is not read (the second step of the product over the column-slab
//    hierarchy, where the "matrix" only lists which partial sums belong to a row).
template <int THREADS, int NPT, int MODE, int VARIANT>
__global__ __launch_bounds__(THREADS) void k_spmv_pos(int rows, int cols, int nnz, const int *__restrict__ pos,
                                                      const int *__restrict__ crd,
                                                      const float *__restrict__ vals,
                                                      const float *__restrict__ x, float *__restrict__ y,
                                                      const int *__restrict__ tile_row,
                                                      int *__restrict__ carry_row,
                                                      float *__restrict__ carry_val, int ntiles, int clo,
                                                      int chi, int accum, const int *__restrict__ rowmap,
                                                      int *__restrict__ tile_cols, int *__restrict__ gap)
{
    constexpr int T = THREADS * NPT;
    constexpr int NW = THREADS / WAVE;
    constexpr int LONG = 32;
    constexpr int MAXLONG = T / LONG;
    constexpr bool VEC = MODE != 0;
    constexpr bool WIN = VARIANT == 1 || VARIANT == 5, ATOM = VARIANT == 2, NOTEMP = VARIANT == 3;
    constexpr bool ROWMAP = VARIANT == 4 || VARIANT == 5;
    constexpr bool ONES = VARIANT == 6;
    constexpr bool SINGLE = VARIANT == 7;
    constexpr bool GAPS = VARIANT == 0 || VARIANT == 1 || VARIANT == 6;   // may leave long runs of empty rows to the fix-up
    static_assert(NPT % 4 == 0, "NPT must be a multiple of 4");
    __shared__ float sprod[skewed_size<1>(T)];
    __shared__ int slong[MAXLONG * 3];
    __shared__ int nlong;
    __shared__ float swave[NW];
    __shared__ int srowid[GAPS ? T : 1];

    const int t = SINGLE ? (blockIdx.x == 0 ? 0 : -1) : xcd_tile(blockIdx.x, ntiles);
    if (t < 0) return;
    PSK_TRACE_WORKGROUP();
    const int tid = threadIdx.x, lane = tid & (WAVE - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / WAVE);   // tells the compiler it is uniform
    const int t0 = t * T;
    const int cnt = (nnz - t0 < T) ? nnz - t0 : T;
    const int t1 = t0 + cnt;

    // A later column pass leaves at once when the first pass found no column of this tile in its window
    // (tiles inside a long sorted row lie in one window only).  The price is one dependent load ahead of
    // the streams for the tiles that stay.
    if (WIN && accum) {
        const v4i a = *reinterpret_cast<const v4i *>(tile_cols + (long long)t * 8);
        const v4i b = *reinterpret_cast<const v4i *>(tile_cols + (long long)t * 8 + 4);
        int mn = a.x < a.z ? a.x : a.z, mx = a.y > a.w ? a.y : a.w;
        mn = b.x < mn ? b.x : mn; mn = b.z < mn ? b.z : mn;
        mx = b.y > mx ? b.y : mx; mx = b.w > mx ? b.w : mx;
        if (mx < clo || mn >= chi) return;
    }

    // Issue order matters more than anything else here: the tile's row bounds hang off a chain of
    // dependent loads (tile_row -> pos), so that chain is started first and runs underneath the
    // streaming loads and the gather instead of after them.
    const int r0 = SINGLE ? 0 : tile_row[t], r1 = SINGLE ? rows : tile_row[t + 1];

    // ---- 1. stream + gather + multiply
    float prod[NPT];
    v4i cv[VEC ? NPT / 4 : 1];
    v4f vv[VEC ? NPT / 4 : 1];
    int cs[MODE == 1 ? 1 : NPT];
    float vs[MODE == 1 ? 1 : NPT];
    const bool full = (cnt == T) && !NOTEMP;
    if (full) {
        if (VEC) {
#pragma unroll
            for (int g = 0; g < NPT / 4; ++g) {
                const int off = t0 + (g * THREADS + tid) * 4;
                cv[g] = ld_stream(reinterpret_cast<const v4i *>(crd + off));
                if (ONES) vv[g] = v4f{1.0f, 1.0f, 1.0f, 1.0f};
                else vv[g] = ld_stream(reinterpret_cast<const v4f *>(vals + off));
            }
        } else {
#pragma unroll
            for (int g = 0; g < NPT; ++g) {
                cs[g] = ld_stream(crd + t0 + g * THREADS + tid);
                vs[g] = ONES ? 1.0f : ld_stream(vals + t0 + g * THREADS + tid);
            }
        }
    }

    // ---- 2. rows of this tile (loads issued before the gather)
    const int p_r0 = pos[r0], p_r1 = pos[r1];
    const int rbeg = (t == 0) ? 0 : r0;
    int my_lo = 0, my_hi = 0;                       // pos pair of the first row this thread will look at
    if (rbeg + tid < rows) {
        my_lo = pos[rbeg + tid];
        my_hi = pos[rbeg + tid + 1];
    }

    if (NOTEMP) {
        if (tid == 0) nlong = 0;
#pragma unroll 1
        for (int g = 0; g < NPT; ++g) {
            const int i = g * THREADS + tid;
            sprod[skew<1>(i)] = i < cnt ? vals[t0 + i] * x[crd[t0 + i]] : 0.0f;
        }
    } else if (full) {
        if (MODE == 1) {
            float xg[NPT / 4][4];
            RunPlan plan[NPT / 4];
            bool ok = true;
#pragma unroll
            for (int g = 0; g < NPT / 4; ++g) {
                plan[g] = run_plan(cv[g], cols);
                ok = ok && plan[g].ok;
            }
            if (WIN) {      // a column pass: only columns in [clo, chi)
#pragma unroll
                for (int g = 0; g < NPT / 4; ++g) {
                    xg[g][0] = (cv[g].x >= clo && cv[g].x < chi) ? x[cv[g].x] : 0.0f;
                    xg[g][1] = (cv[g].y >= clo && cv[g].y < chi) ? x[cv[g].y] : 0.0f;
                    xg[g][2] = (cv[g].z >= clo && cv[g].z < chi) ? x[cv[g].z] : 0.0f;
                    xg[g][3] = (cv[g].w >= clo && cv[g].w < chi) ? x[cv[g].w] : 0.0f;
                }
            } else if (__ballot(!ok) == 0ull) {
                v4f_u wA[NPT / 4], wB[NPT / 4];
#pragma unroll
                for (int g = 0; g < NPT / 4; ++g) {
                    wA[g] = *reinterpret_cast<const v4f_u *>(x + cv[g].x);
                    wB[g] = *reinterpret_cast<const v4f_u *>(x + plan[g].colB);
                }
#pragma unroll
                for (int g = 0; g < NPT / 4; ++g) run_select(plan[g], wA[g], wB[g], xg[g]);
            } else {
#pragma unroll
                for (int g = 0; g < NPT / 4; ++g) {
                    xg[g][0] = x[cv[g].x];
                    xg[g][1] = x[cv[g].y];
                    xg[g][2] = x[cv[g].z];
                    xg[g][3] = x[cv[g].w];
                }
            }
#pragma unroll
            for (int g = 0; g < NPT / 4; ++g) {
                prod[4 * g + 0] = vv[g].x * xg[g][0];
                prod[4 * g + 1] = vv[g].y * xg[g][1];
                prod[4 * g + 2] = vv[g].z * xg[g][2];
                prod[4 * g + 3] = vv[g].w * xg[g][3];
            }
        } else {
#pragma unroll
            for (int g = 0; g < NPT; ++g)
                prod[g] = (!WIN || (cs[g] >= clo && cs[g] < chi)) ? vs[g] * x[cs[g]] : 0.0f;
        }
    } else {   // last tile: guarded
#pragma unroll
        for (int g = 0; g < NPT; ++g) {
            const int i = tile_index<MODE, THREADS>(g, tid);
            float pr = 0.0f;
            if (i < cnt) {
                const int c = crd[t0 + i];
                if (!WIN || (c >= clo && c < chi)) pr = ONES ? x[c] : vals[t0 + i] * x[c];
            }
            prod[g] = pr;
        }
    }

    if (WIN && !accum) {    // first column pass: leave the tile's column range for the later ones
        int mn = 0x7fffffff, mx = -1;
        if (full) {
            if (MODE == 1) {
#pragma unroll
                for (int g = 0; g < NPT / 4; ++g) {
                    const int lo4 = min(min(cv[g].x, cv[g].y), min(cv[g].z, cv[g].w));
                    const int hi4 = max(max(cv[g].x, cv[g].y), max(cv[g].z, cv[g].w));
                    mn = min(mn, lo4);
                    mx = max(mx, hi4);
                }
            } else {
#pragma unroll
                for (int g = 0; g < NPT; ++g) { mn = min(mn, cs[g]); mx = max(mx, cs[g]); }
            }
        } else {
#pragma unroll
            for (int g = 0; g < NPT; ++g) {
                const int i = tile_index<MODE, THREADS>(g, tid);
                if (i < cnt) { const int c = crd[t0 + i]; mn = min(mn, c); mx = max(mx, c); }
            }
        }
#pragma unroll
        for (int m = 1; m < WAVE; m <<= 1) {
            mn = min(mn, __shfl_xor(mn, m, WAVE));
            mx = max(mx, __shfl_xor(mx, m, WAVE));
        }
        if (lane == 0) {
            tile_cols[(long long)t * 8 + 2 * wave] = mn;
            tile_cols[(long long)t * 8 + 2 * wave + 1] = mx;
        }
        if (tid < 2 * (4 - NW)) tile_cols[(long long)t * 8 + 2 * NW + tid] = (tid & 1) ? -1 : 0x7fffffff;
    }

    const bool has_carry = (t > 0) && (p_r0 < t0);
    const int rend = (p_r1 == t1) ? r1 : r1 + 1;   // last tile: r1 = rows and pos[rows] = nnz = t1
    if (tid == 0 && !has_carry && !ATOM && !SINGLE) carry_row[t] = -1;
    // a later column pass adds to what the first one stored (same lane, same order: deterministic)
    auto emit = [&](int r, float v) {
        if (ATOM) {
            // the schedule's own race strategy (appendix "SPMV on a GPU": Atomics): y was zero-filled;
            // a row that other tiles also hold part of is added atomically, the rest is stored
            if ((has_carry && r == r0) || (p_r1 != t1 && r == r1)) unsafeAtomicAdd(&y[r], v);
            else y[r] = v;
            return;
        }
        if (has_carry && r == r0) {
            carry_row[t] = r;
            carry_val[t] = (WIN && accum) ? carry_val[t] + v : v;
        } else if (ROWMAP) {
            float *dst = y + rowmap[r];
            *dst = (WIN && accum) ? *dst + v : v;
        } else {
            y[r] = (WIN && accum) ? y[r] + v : v;
        }
    };

    // ---- 3a. the tile lies inside a single row
    if (!NOTEMP && rend - rbeg == 1) {
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
            emit(rbeg, tot);
        }
        return;
    }

    // ---- 3b. several rows: products to LDS in position order
    if (!NOTEMP) {
        if (tid == 0) nlong = 0;
#pragma unroll
        for (int g = 0; g < NPT; ++g) sprod[skew<1>(tile_index<MODE, THREADS>(g, tid))] = prod[g];
    }
    __syncthreads();
    if (GAPS && gap && rend - rbeg > kGapRows) {
        // The tile's rows span a long run of empty rows (Section 6.2 walks past empty rows one by one; here that walk
        // would be done by this one workgroup).  Instead the row of every position is found by search -- a thread takes
        // NPT consecutive positions, searches once for the first and again whenever a row ends --, the row segments
        // are summed by the thread that holds their first position, and the run of rows is handed to the fix-up step,
        // whose extra workgroups clear its empty rows at full width.
        const int i0 = tid * NPT;
        if (i0 < cnt) {
            int lo = r0, hi = r1;                       // max { r in [r0, r1] : pos[r] <= t0 + i0 }
            while (lo < hi) {
                const int mid = lo + ((hi - lo + 1) >> 1);
                if (pos[mid] <= t0 + i0) lo = mid; else hi = mid - 1;
            }
            int r = lo;
            int next = pos[r + 1];
#pragma unroll 1
            for (int k = 0; k < NPT && i0 + k < cnt; ++k) {
                const int p = t0 + i0 + k;
                if (p >= next) {                        // the row ended: the next row with entries owns p
                    int l2 = r + 1, h2 = r1;
                    while (l2 < h2) {
                        const int mid = l2 + ((h2 - l2 + 1) >> 1);
                        if (pos[mid] <= p) l2 = mid; else h2 = mid - 1;
                    }
                    r = l2;
                    next = pos[r + 1];
                }
                srowid[i0 + k] = r;
            }
        }
        __syncthreads();
#pragma unroll 1
        for (int k = 0; k < NPT && i0 + k < cnt; ++k) {
            const int i = i0 + k;
            const int r = srowid[i];
            if (i > 0 && srowid[i - 1] == r) continue;  // not the first position of its row segment
            float sum = 0.0f;
            for (int j = i; j < cnt && srowid[j] == r; ++j) sum += sprod[skew<1>(j)];
            emit(r, sum);
        }
        if (tid == 0 && !(WIN && accum)) {
            const int e = atomicAdd(&gap[0], 1);
            if (e < ntiles) { gap[2 + 2 * e] = rbeg; gap[3 + 2 * e] = rend; }
        }
        return;
    }
    for (int r = rbeg + tid; r < rend; r += THREADS) {
        int lo = my_lo - t0, hi = my_hi - t0;
        if (r + THREADS < rend) { my_lo = pos[r + THREADS]; my_hi = pos[r + THREADS + 1]; }
        lo = lo < 0 ? 0 : lo;
        hi = hi > cnt ? cnt : hi;
        if (hi - lo < LONG) {
            // serial, in position order; four reads are issued before their adds so that the LDS
            // latency is paid once per four elements
            float s = 0.0f;
            int i = lo;
            for (; i + 4 <= hi; i += 4) {
                const float a = sprod[skew<1>(i)], b = sprod[skew<1>(i + 1)], c = sprod[skew<1>(i + 2)],
                            d = sprod[skew<1>(i + 3)];
                s += a; s += b; s += c; s += d;
            }
            for (; i < hi; ++i) s += sprod[skew<1>(i)];
            emit(r, s);
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
        if (lane == 0) emit(r, s);
    }
}

bool spmv_csr_tile_ok(int32_t tile)
{
    return tile == 256 || tile == 512 || tile == 1024 || tile == 2048 || tile == 4096;
}

template <int THREADS, int NPT>
static void launch_pos(int mode, int grid, hipStream_t s, int rows, int cols, int nnz, const int *pos, const int *crd,
                       const float *vals, const float *x, float *y, const Workspace &w, int ntiles, int clo, int chi,
                       int accum, const int *rowmap, int *gap)
{
#define PSK_GO(M, W)                                                                                             \
    PSK_LAUNCH((k_spmv_pos<THREADS, NPT, M, W>), dim3(grid), dim3(THREADS), 0, s, rows, cols, nnz, pos,  \
                       crd, vals, x, y, w.tile_row, w.carry_row, w.carry_val, ntiles, clo, chi, accum, rowmap,    \
                       w.tile_cols, gap)
    const bool window = clo > 0 || chi < cols;
    const int variant = rowmap ? (window ? 5 : 4) : (accum >= 2 ? accum : (window ? 1 : 0));
    if (variant == 3) PSK_GO(0, 3);
    else if (variant == 4) { if (mode == 1) PSK_GO(1, 4); else PSK_GO(0, 4); }
    else if (variant == 5) { if (mode == 1) PSK_GO(1, 5); else PSK_GO(0, 5); }
    else if (mode == 1) { if (variant == 2) PSK_GO(1, 2); else if (variant == 1) PSK_GO(1, 1); else PSK_GO(1, 0); }
    else { if (variant == 2) PSK_GO(0, 2); else if (variant == 1) PSK_GO(0, 1); else PSK_GO(0, 0); }
#undef PSK_GO
}

// nnz <= kSingleTile: the whole product in one launch of one workgroup
hipError_t launch_spmv_csr_single(int32_t rows, int32_t cols, int32_t nnz, const int32_t *pos, const int32_t *crd,
                                  const float *vals, const float *x, float *y, hipStream_t s)
{
    if (nnz <= 0 || nnz > kSingleTile) return hipErrorInvalidValue;
    const int *notable = nullptr;
    int *nocarry = nullptr;
    float *nocarryval = nullptr;
    const bool aligned = ((reinterpret_cast<uintptr_t>(crd) | reinterpret_cast<uintptr_t>(vals)) & 15) == 0;
    if (aligned)
        PSK_LAUNCH((k_spmv_pos<1024, 16, 1, 7>), dim3(1), dim3(1024), 0, s, rows, cols, nnz, pos, crd, vals, x, y, notable,
                   nocarry, nocarryval, 1, 0, cols, 0, notable, nocarry, nocarry);
    else
        PSK_LAUNCH((k_spmv_pos<1024, 16, 0, 7>), dim3(1), dim3(1024), 0, s, rows, cols, nnz, pos, crd, vals, x, y, notable,
                   nocarry, nocarryval, 1, 0, cols, 0, notable, nocarry, nocarry);
    return take_launch_status();
}

hipError_t launch_spmv_csr_ones(int32_t rows, int32_t cols, int32_t nnz, const int32_t *pos, const int32_t *crd,
                                const float *x, float *y, const Workspace &w, hipStream_t s)
{
    const int ntiles = (int)(((int64_t)nnz + 2047) / 2048);
    if (ntiles == 0) return hipSuccess;
    const int grid = xcd_grid(ntiles);
    const float *none = nullptr;
    const int *nomap = nullptr;
    if ((reinterpret_cast<uintptr_t>(crd) & 15) == 0)
        PSK_LAUNCH((k_spmv_pos<256, 8, 1, 6>), dim3(grid), dim3(256), 0, s, rows, cols, nnz, pos, crd, none, x, y,
                   w.tile_row, w.carry_row, w.carry_val, ntiles, 0, cols, 0, nomap, w.tile_cols, w.gap);
    else
        PSK_LAUNCH((k_spmv_pos<256, 8, 0, 6>), dim3(grid), dim3(256), 0, s, rows, cols, nnz, pos, crd, none, x, y,
                   w.tile_row, w.carry_row, w.carry_val, ntiles, 0, cols, 0, nomap, w.tile_cols, w.gap);
    return take_launch_status();
}

hipError_t launch_spmv_csr_main(int32_t rows, int32_t cols, int32_t nnz, const int32_t *pos, const int32_t *crd,
                                const float *vals, const float *x, float *y, int32_t tile, int32_t col_passes,
                                const Workspace &w, hipStream_t s, const int32_t *rowmap, bool gaps)
{
    const int ntiles = (int)(((int64_t)nnz + tile - 1) / tile);
    if (ntiles == 0) return hipSuccess;
    const int grid = xcd_grid(ntiles);
    int *gap = gaps ? w.gap : nullptr;
    // baselines: -1 = one pass with atomic adds for rows that span tiles, -2 = one pass without the
    // register temporary and the unrolled load loop
    const int baseline = col_passes == -1 ? 2 : (col_passes == -2 ? 3 : 0);
    if (col_passes < 1) col_passes = 1;
    for (int p = 0; p < col_passes; ++p) {
    const int clo = (int)((int64_t)cols * p / col_passes), chi = (int)((int64_t)cols * (p + 1) / col_passes);
    const int accum = baseline ? baseline : (p > 0);
    const bool aligned = ((reinterpret_cast<uintptr_t>(crd) | reinterpret_cast<uintptr_t>(vals)) & 15) == 0;
    const int vec = aligned ? 1 : 0;
    switch (tile) {
        case 256:  launch_pos<64, 4>(vec, grid, s, rows, cols, nnz, pos, crd, vals, x, y, w, ntiles, clo, chi, accum, rowmap, gap); break;
        case 512:  launch_pos<128, 4>(vec, grid, s, rows, cols, nnz, pos, crd, vals, x, y, w, ntiles, clo, chi, accum, rowmap, gap); break;
        case 1024: launch_pos<256, 4>(vec, grid, s, rows, cols, nnz, pos, crd, vals, x, y, w, ntiles, clo, chi, accum, rowmap, gap); break;
        case 2048: launch_pos<256, 8>(vec, grid, s, rows, cols, nnz, pos, crd, vals, x, y, w, ntiles, clo, chi, accum, rowmap, gap); break;
        case 4096: launch_pos<256, 16>(vec, grid, s, rows, cols, nnz, pos, crd, vals, x, y, w, ntiles, clo, chi, accum, rowmap, gap); break;
        default: return hipErrorInvalidValue;
    }
    }
    return take_launch_status();
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
    PSK_TRACE_WORKGROUP();
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
                                                           float *__restrict__ y,
                                                           const int *__restrict__ rowmap)
{
    PSK_TRACE_WORKGROUP();
    const int lane = threadIdx.x & (WAVE - 1);
    const int r = blockIdx.x * (256 / WAVE) + threadIdx.x / WAVE;
    if (r >= rows) return;
    const int pe = pos[r + 1];
    float s = 0.0f;
    for (int p = pos[r] + lane; p < pe; p += WAVE) s += vals[p] * x[crd[p]];
    s = wave_sum(s);
    if (lane == 0) y[rowmap ? rowmap[r] : r] = s;
}

hipError_t launch_spmv_rowsplit(int32_t rows, const int32_t *pos, const int32_t *crd, const float *vals,
                                const float *x, float *y, int variant, hipStream_t s, const int32_t *rowmap)
{
    if (rows == 0) return hipSuccess;
    if (variant == 0)
        PSK_LAUNCH(k_spmv_thread_per_row, dim3((rows + 255) / 256), dim3(256), 0, s, rows, pos, crd, vals, x,
                           y);
    else
        PSK_LAUNCH(k_spmv_wave_per_row, dim3((rows + 3) / 4), dim3(256), 0, s, rows, pos, crd, vals, x, y,
                           rowmap);
    return take_launch_status();
}

#ifdef PSK_CU_TRACE
hipError_t cu_trace_set_spmv_csr(void *buf, unsigned records) { return cu_trace_set_here(buf, records); }
#endif

}  // namespace psk
