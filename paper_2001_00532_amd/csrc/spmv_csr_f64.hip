// CSR SpMV with fp64 values, vector and result: the value type of the paper's own schedules (the
// per-thread temporary of appendix "SPMV on a GPU" is declared Float64).  Same position cut, row
// logic and carry records as the fp32 kernel; one pass, 8-byte gathers.
#include "psk_dev.h"
#include "psk_internal.h"

namespace psk {

typedef double v2d __attribute__((ext_vector_type(2)));

// Sum over the 64 lanes of a wave, same bits in every lane (xor butterfly through the LDS crossbar).
__device__ __forceinline__ double wave_sum_f64(double v)
{
#pragma unroll
    for (int m = 1; m < WAVE; m <<= 1) v += __shfl_xor(v, m, WAVE);
    return v;
}

// One workgroup per tile of T = THREADS*NPT positions.  VEC: crd is read with 16-byte loads and vals
// with two 16-byte loads per four positions (both arrays 16-byte aligned), a lane keeps four
// consecutive positions; otherwise 4- and 8-byte loads at lane-consecutive positions.
// WIN: a column pass as in the fp32 kernel: only columns in [clo, chi) contribute, accum adds to what the
// earlier passes stored; the first pass records the tile's column range, later passes skip tiles outside
// their window.
// ONES: every stored value is 1 and `vals` is not read (the row sums over the pair array of the slab path).
template <int THREADS, int NPT, bool VEC, bool WIN, bool ONES = false>
__global__ __launch_bounds__(THREADS) void k_spmv_pos_f64(int rows, int nnz, const int *__restrict__ pos,
                                                          const int *__restrict__ crd,
                                                          const double *__restrict__ vals,
                                                          const double *__restrict__ x, double *__restrict__ y,
                                                          const int *__restrict__ tile_row,
                                                          int *__restrict__ carry_row,
                                                          double *__restrict__ carry_val, int ntiles, int clo,
                                                          int chi, int accum, int *__restrict__ tile_cols,
                                                          int *__restrict__ gap)
{
    constexpr int T = THREADS * NPT;
    constexpr int NW = THREADS / WAVE;
    constexpr int LONG = 32;
    constexpr int MAXLONG = T / LONG;
    static_assert(NPT % 4 == 0, "NPT must be a multiple of 4");
    __shared__ double sprod[skewed_size<1>(T)];
    __shared__ int slong[MAXLONG * 3];
    __shared__ int nlong;
    __shared__ double swave[NW];
    __shared__ int srowid[T];            // row of every position of the tile (only when the tile spans a long run of empty rows)

    const int t = xcd_tile(blockIdx.x, ntiles);
    if (t < 0) return;
    const int tid = threadIdx.x, lane = tid & (WAVE - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / WAVE);
    const int t0 = t * T;
    const int cnt = (nnz - t0 < T) ? nnz - t0 : T;
    const int t1 = t0 + cnt;
    auto index = [&](int g) { return VEC ? ((g / 4) * THREADS + tid) * 4 + (g & 3) : g * THREADS + tid; };

    if (WIN && accum) {
        const v4i a = *reinterpret_cast<const v4i *>(tile_cols + (long long)t * 8);
        const v4i b = *reinterpret_cast<const v4i *>(tile_cols + (long long)t * 8 + 4);
        int mn = a.x < a.z ? a.x : a.z, mx = a.y > a.w ? a.y : a.w;
        mn = b.x < mn ? b.x : mn; mn = b.z < mn ? b.z : mn;
        mx = b.y > mx ? b.y : mx; mx = b.w > mx ? b.w : mx;
        if (mx < clo || mn >= chi) return;
    }

    // the dependent chain tile_row -> pos is started first and runs underneath the streams
    const int r0 = tile_row[t], r1 = tile_row[t + 1];

    double prod[NPT];
    int cmin = 0x7fffffff, cmax = -1;             // column range of the tile (first column pass)
    const bool full = cnt == T;
    if (full) {
        int c[NPT];
        double v[NPT];
        if (VEC) {
#pragma unroll
            for (int g = 0; g < NPT / 4; ++g) {
                const int off = t0 + (g * THREADS + tid) * 4;
                const v4i cv = ld_stream(reinterpret_cast<const v4i *>(crd + off));
                v2d va = {1.0, 1.0}, vb = {1.0, 1.0};
                if (!ONES) {
                    va = ld_stream(reinterpret_cast<const v2d *>(vals + off));
                    vb = ld_stream(reinterpret_cast<const v2d *>(vals + off + 2));
                }
                c[4 * g] = cv.x; c[4 * g + 1] = cv.y; c[4 * g + 2] = cv.z; c[4 * g + 3] = cv.w;
                v[4 * g] = va.x; v[4 * g + 1] = va.y; v[4 * g + 2] = vb.x; v[4 * g + 3] = vb.y;
            }
        } else {
#pragma unroll
            for (int g = 0; g < NPT; ++g) {
                c[g] = ld_stream(crd + t0 + g * THREADS + tid);
                v[g] = ONES ? 1.0 : ld_stream(vals + t0 + g * THREADS + tid);
            }
        }
        double xg[NPT];
#pragma unroll
        for (int g = 0; g < NPT; ++g) xg[g] = (!WIN || (c[g] >= clo && c[g] < chi)) ? x[c[g]] : 0.0;
#pragma unroll
        for (int g = 0; g < NPT; ++g) prod[g] = v[g] * xg[g];
        if (WIN && !accum) {
#pragma unroll
            for (int g = 0; g < NPT; ++g) { cmin = min(cmin, c[g]); cmax = max(cmax, c[g]); }
        }
    }

    const int p_r0 = pos[r0], p_r1 = pos[r1];
    const int rbeg = (t == 0) ? 0 : r0;
    int my_lo = 0, my_hi = 0;
    if (rbeg + tid < rows) {
        my_lo = pos[rbeg + tid];
        my_hi = pos[rbeg + tid + 1];
    }

    if (!full) {   // last tile: guarded
#pragma unroll
        for (int g = 0; g < NPT; ++g) {
            const int i = index(g);
            double pr = 0.0;
            if (i < cnt) {
                const int c = crd[t0 + i];
                cmin = min(cmin, c);
                cmax = max(cmax, c);
                if (!WIN || (c >= clo && c < chi)) pr = ONES ? x[c] : vals[t0 + i] * x[c];
            }
            prod[g] = pr;
        }
    }
    if (WIN && !accum) {
#pragma unroll
        for (int m = 1; m < WAVE; m <<= 1) {
            cmin = min(cmin, __shfl_xor(cmin, m, WAVE));
            cmax = max(cmax, __shfl_xor(cmax, m, WAVE));
        }
        if (lane == 0) {
            tile_cols[(long long)t * 8 + 2 * wave] = cmin;
            tile_cols[(long long)t * 8 + 2 * wave + 1] = cmax;
        }
        if (tid < 2 * (4 - NW)) tile_cols[(long long)t * 8 + 2 * NW + tid] = (tid & 1) ? -1 : 0x7fffffff;
    }

    const bool has_carry = (t > 0) && (p_r0 < t0);
    const int rend = (p_r1 == t1) ? r1 : r1 + 1;
    if (tid == 0 && !has_carry) carry_row[t] = -1;
    auto emit = [&](int r, double v) {
        if (has_carry && r == r0) {
            carry_row[t] = r;
            carry_val[t] = (WIN && accum) ? carry_val[t] + v : v;
        } else {
            y[r] = (WIN && accum) ? y[r] + v : v;
        }
    };

    if (rend - rbeg == 1) {   // the tile lies inside a single row
        double s = 0.0;
#pragma unroll
        for (int g = 0; g < NPT; ++g) s += prod[g];
        s = wave_sum_f64(s);
        if (lane == 0) swave[wave] = s;
        __syncthreads();
        if (tid == 0) {
            double tot = swave[0];
#pragma unroll
            for (int w = 1; w < NW; ++w) tot += swave[w];
            emit(rbeg, tot);
        }
        return;
    }

    if (tid == 0) nlong = 0;
#pragma unroll
    for (int g = 0; g < NPT; ++g) sprod[skew<1>(index(g))] = prod[g];
    __syncthreads();
    if (gap && rend - rbeg > kGapRows) {
        // The tile's rows span a long run of empty rows (Section 6.2 walks past empty rows one by one; here that walk
        // would be done by this one workgroup).  As in the fp32 kernel: the row of every position is found by search (a
        // thread takes NPT consecutive positions), the row segments are summed by the thread that holds their first
        // position, and the run of rows is handed to the fix-up step, whose extra workgroups clear its empty rows.
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
            double sum = 0.0;
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
            double s = 0.0;
            int i = lo;
            for (; i + 4 <= hi; i += 4) {
                const double a = sprod[skew<1>(i)], b = sprod[skew<1>(i + 1)], c = sprod[skew<1>(i + 2)],
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
        double s = 0.0;
        for (int i = lo + lane; i < hi; i += WAVE) s += sprod[skew<1>(i)];
        s = wave_sum_f64(s);
        if (lane == 0) emit(r, s);
    }
}

bool spmv_csr_f64_tile_ok(int32_t tile) { return tile == 256 || tile == 512 || tile == 1024 || tile == 2048; }

template <int THREADS, int NPT>
static void go(bool vec, bool win, int grid, hipStream_t s, int rows, int nnz, const int *pos, const int *crd,
               const double *vals, const double *x, double *y, const Workspace &w, int ntiles, int clo, int chi, int accum,
               int *gap)
{
    double *cv = reinterpret_cast<double *>(w.carry_val);
#define PSK_GO(V, W)                                                                                                  \
    PSK_LAUNCH((k_spmv_pos_f64<THREADS, NPT, V, W>), dim3(grid), dim3(THREADS), 0, s, rows, nnz, pos, crd, vals, \
                       x, y, w.tile_row, w.carry_row, cv, ntiles, clo, chi, accum, w.tile_cols, gap)
    if (vec) { if (win) PSK_GO(true, true); else PSK_GO(true, false); }
    else { if (win) PSK_GO(false, true); else PSK_GO(false, false); }
#undef PSK_GO
}

hipError_t launch_spmv_csr_f64_main(int32_t rows, int32_t cols, int32_t nnz, const int32_t *pos, const int32_t *crd,
                                    const double *vals, const double *x, double *y, int32_t tile, int32_t col_passes,
                                    const Workspace &w, hipStream_t s, bool gaps)
{
    int *gap = gaps ? w.gap : nullptr;
    const int ntiles = (int)(((int64_t)nnz + tile - 1) / tile);
    if (ntiles == 0) return hipSuccess;
    const int grid = xcd_grid(ntiles);
    const bool vec = ((reinterpret_cast<uintptr_t>(crd) | reinterpret_cast<uintptr_t>(vals)) & 15) == 0;
    if (col_passes < 1) col_passes = 1;
    for (int p = 0; p < col_passes; ++p) {
        const int clo = (int)((int64_t)cols * p / col_passes), chi = (int)((int64_t)cols * (p + 1) / col_passes);
        const bool win = col_passes > 1;
        const int accum = p > 0;
        switch (tile) {
            case 256:  go<64, 4>(vec, win, grid, s, rows, nnz, pos, crd, vals, x, y, w, ntiles, clo, chi, accum, gap); break;
            case 512:  go<128, 4>(vec, win, grid, s, rows, nnz, pos, crd, vals, x, y, w, ntiles, clo, chi, accum, gap); break;
            case 1024: go<256, 4>(vec, win, grid, s, rows, nnz, pos, crd, vals, x, y, w, ntiles, clo, chi, accum, gap); break;
            case 2048: go<256, 8>(vec, win, grid, s, rows, nnz, pos, crd, vals, x, y, w, ntiles, clo, chi, accum, gap); break;
            default: return hipErrorInvalidValue;
        }
    }
    return take_launch_status();
}

// y = Q * P with unit values over (pos, crd) = the row lists of the slab structure; tile 1024 or 2048
hipError_t launch_spmv_csr_f64_ones(int32_t rows, int32_t nnz, const int32_t *pos, const int32_t *crd, const double *x,
                                    double *y, int32_t tile, const Workspace &w, hipStream_t s)
{
    if (tile != 1024 && tile != 2048) return hipErrorInvalidValue;
    const int ntiles = (int)(((int64_t)nnz + tile - 1) / tile);
    if (ntiles == 0) return hipSuccess;
    const int grid = xcd_grid(ntiles);
    const double *none = nullptr;
    double *cv = reinterpret_cast<double *>(w.carry_val);
    const bool vec = (reinterpret_cast<uintptr_t>(crd) & 15) == 0;
#define PSK_GO(NPT, V)                                                                                                   \
    PSK_LAUNCH((k_spmv_pos_f64<256, NPT, V, false, true>), dim3(grid), dim3(256), 0, s, rows, nnz, pos, crd, none, x, y, \
               w.tile_row, w.carry_row, cv, ntiles, 0, 0x7fffffff, 0, w.tile_cols, w.gap)
    if (tile == 2048) { if (vec) PSK_GO(8, true); else PSK_GO(8, false); }
    else { if (vec) PSK_GO(4, true); else PSK_GO(4, false); }
#undef PSK_GO
    return take_launch_status();
}

}  // namespace psk
