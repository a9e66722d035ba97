// CSR SpMM for narrow dense operands (k <= 32).  The SpMM kernel maps the 64 lanes of a wave to 64*VEC
// columns of B; with k <= 32 half or more of the lanes would idle and every load instruction would fetch
// one row of <= 128 bytes.  Here the wave is split into G = 2, 4 or 8 groups of 64/G lanes; in one step the
// groups take G consecutive positions (group g the g-th), so a load instruction fetches G rows of B.  Every
// lane keeps the partial sum of its group for the open row; at a row end the partial sums of the groups
// are added through the LDS crossbar.  Cut, row-end flags, records, carries: as in the SpMM kernel.
#include "psk_dev.h"
#include "psk_internal.h"

namespace psk {

template <int G>
__global__ __launch_bounds__(256) void k_spmm_pos_narrow(int rows, int nnz, const int *__restrict__ pos,
                                                         const int *__restrict__ crd,
                                                         const float *__restrict__ vals,
                                                         const float *__restrict__ B, int k, long long ldb,
                                                         float *__restrict__ C, long long ldc,
                                                         const int *__restrict__ tile_row,
                                                         int *__restrict__ carry_row,
                                                         float *__restrict__ carry_val, int ntiles, int T)
{
    constexpr int THREADS = 256, NW = THREADS / WAVE, GW = WAVE / G, U = 4;
    extern __shared__ int sflag[];                // T ints
    __shared__ float srec[2 * NW][GW];
    __shared__ int srec_row[2 * NW];              // -2 unused, -1 open segment, >= 0 row that ended

    const int t = xcd_tile(blockIdx.x, ntiles);
    if (t < 0) return;
    const int tid = threadIdx.x, lane = tid & (WAVE - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / WAVE);
    const int g = lane / GW, col = lane % GW;
    const bool active = col < k;
    const bool writer = active && g == 0;         // group 0 stores on behalf of the wave
    const int lcol = active ? col : 0;
    const int t0 = t * T;
    const int cnt = (nnz - t0 < T) ? nnz - t0 : T;
    const int t1 = t0 + cnt;

    for (int i = tid; i < T; i += THREADS) sflag[i] = -1;
    if (tid < 2 * NW) srec_row[tid] = -2;

    const int r0 = tile_row[t], r1 = tile_row[t + 1];
    const bool has_carry = (t > 0) && (pos[r0] < t0);
    const int rbeg = (t == 0) ? 0 : r0;
    const bool straddle = pos[r1] != t1;
    const int rend = straddle ? r1 + 1 : r1;
    if (tid == 0 && !has_carry) carry_row[t] = -1;
    __syncthreads();

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
            if (writer) __builtin_nontemporal_store(0.0f, C + (long long)(rb + j) * ldc + col);
        }
    }
    __syncthreads();

    const int CH = T / NW;
    const int wbeg = wave * CH < cnt ? wave * CH : cnt;
    const int wend = wbeg + CH < cnt ? wbeg + CH : cnt;
    float acc = 0.0f;                             // this group's share of the open row
    bool seen = false;

    auto group_sum = [&](float v) {
#pragma unroll
        for (int m = GW; m < WAVE; m <<= 1) v += __shfl_xor(v, m, WAVE);
        return v;
    };
    auto flush = [&](int f, float total) {
        if (!seen) {
            seen = true;
            if (g == 0) srec[2 * wave][col] = total;
            if (lane == 0) srec_row[2 * wave] = f;
        } else if (writer) {
            __builtin_nontemporal_store(total, C + (long long)f * ldc + col);
        }
    };

    int c_n = 0;
    float v_n = 0.0f;
    auto fetch = [&](int base) {
        c_n = 0;
        v_n = 0.0f;
        if (base + lane < wend) {
            c_n = ld_stream(crd + t0 + base + lane);
            v_n = ld_stream(vals + t0 + base + lane);
        }
    };
    fetch(wbeg);
    for (int base = wbeg; base < wend; base += WAVE) {
        const int n = wend - base < WAVE ? wend - base : WAVE;
        const int c_l = c_n;
        const float v_l = v_n;
        const int f_l = lane < n ? sflag[base + lane] : -1;
        fetch(base + WAVE);
        for (int j0 = 0; j0 < n; j0 += U * G) {
            float b[U], a[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int jj = (j0 + u * G + g) & (WAVE - 1);      // this group's position in step u
                const long long c = __shfl(c_l, jj, WAVE);         // lanes past n hold column 0, value 0
                a[u] = __shfl(v_l, jj, WAVE);
                b[u] = B[c * ldb + lcol];
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int s0 = j0 + u * G;                          // first position of the step
                if (s0 < n) {
                    const float term = (s0 + g < n) ? a[u] * b[u] : 0.0f;
                    bool added = false;
#pragma unroll
                    for (int e = 0; e < G; ++e) {
                        const int f = rl(f_l, (s0 + e) & (WAVE - 1));
                        if (f >= 0) {                               // position s0 + e ends row f
                            const bool mine = !added && g <= e;
                            const float total = group_sum(mine ? acc + term : acc);
                            added = added || g <= e;
                            flush(f, total);
                            acc = 0.0f;
                        }
                    }
                    if (!added) acc += term;
                }
            }
        }
    }
    if (wbeg < wend) {
        const float total = group_sum(acc);
        const int slot = seen ? 2 * wave + 1 : 2 * wave;
        if (g == 0) srec[slot][col] = total;
        if (lane == 0) srec_row[slot] = -1;
    }
    __syncthreads();

    if (wave != 0 || g != 0) return;
    float run = 0.0f;
    auto finalize = [&](int r) {
        if (has_carry && r == r0) {
            if (active) carry_val[(long long)t * k + col] = run;
            if (lane == 0) carry_row[t] = r;
        } else if (active) {
            __builtin_nontemporal_store(run, C + (long long)r * ldc + col);
        }
        run = 0.0f;
    };
    for (int rec = 0; rec < 2 * NW; ++rec) {
        const int code = srec_row[rec];
        if (code == -2) continue;
        run += srec[rec][col];
        if (code >= 0) finalize(code);
    }
    if (straddle) finalize(r1);
}

hipError_t launch_spmm_csr_narrow(int32_t rows, int32_t nnz, const int32_t *pos, const int32_t *crd,
                                  const float *vals, const float *B, int32_t k, int64_t ldb, float *C, int64_t ldc,
                                  int32_t tile, const Workspace &w, hipStream_t s)
{
    const int ntiles = (int)(((int64_t)nnz + tile - 1) / tile);
    if (ntiles == 0) return hipSuccess;
    const dim3 grid(xcd_grid(ntiles));
    const size_t lds = (size_t)tile * sizeof(int);
#define PSK_GO(GG)                                                                                               \
    PSK_LAUNCH((k_spmm_pos_narrow<GG>), grid, dim3(256), lds, s, rows, nnz, pos, crd, vals, B, k,        \
                       (long long)ldb, C, (long long)ldc, w.tile_row, w.carry_row, w.carry_val, ntiles, tile)
    if (k <= 8) PSK_GO(8);
    else if (k <= 16) PSK_GO(4);
    else if (k <= 32) PSK_GO(2);
    else return hipErrorInvalidValue;
#undef PSK_GO
    return take_launch_status();
}

}  // namespace psk
