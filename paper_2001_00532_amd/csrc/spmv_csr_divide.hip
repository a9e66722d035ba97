// CSR SpMV with the position space DIVIDED into a fixed number of parts (Section 5 "Divide": the outer
// extent is constant, so the number of searches does not grow with the tensor) instead of split into
// tiles of a fixed size.  One persistent workgroup per part: it finds its first row with one binary
// search over pos (Section 6.2), then walks its part in chunks of T positions and tracks the rows from
// chunk to chunk (the "advance when the end of a row segment is reached" of Section 6.2, done by the
// whole workgroup: the rows of a chunk are scanned 256 at a time until one lies beyond the chunk).
// There is no tile->row table and no partition kernel.  A row that continues into the next chunk of the
// same part is carried in on-chip memory; a row that began in an earlier part goes to the part's carry
// record, exactly as in the tiled kernel, and the same fix-up adds the records.
#include "psk_dev.h"
#include "psk_internal.h"

namespace psk {

template <int THREADS, int NPT, bool VEC>
__global__ __launch_bounds__(THREADS) void k_spmv_div(int rows, int cols, int nnz, const int *__restrict__ pos,
                                                      const int *__restrict__ crd,
                                                      const float *__restrict__ vals,
                                                      const float *__restrict__ x, float *__restrict__ y,
                                                      int *__restrict__ carry_row,
                                                      float *__restrict__ carry_val, int chunks_per_part)
{
    constexpr int T = THREADS * NPT;
    constexpr int NW = THREADS / WAVE;
    constexpr int LONG = 32;
    constexpr int MAXLONG = T / LONG;
    static_assert(NPT % 4 == 0, "NPT must be a multiple of 4");
    __shared__ float sprod[skewed_size<1>(T)];
    __shared__ int slong[MAXLONG * 4];
    __shared__ int nlong;
    __shared__ int s_next;            // max row index i seen with pos[i] <= end of the chunk
    __shared__ float s_pend[2];       // partial sum of the row that continues into the next chunk

    const int p = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & (WAVE - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / WAVE);
    const long long part_len = (long long)chunks_per_part * T;
    const long long b0l = p * part_len;
    if (b0l >= nnz) {                 // cannot happen with the launcher's grid; keeps the record defined
        if (tid == 0) carry_row[p] = -1;
        return;
    }
    const int b0 = (int)b0l;
    const int b1 = (b0l + part_len < nnz) ? (int)(b0l + part_len) : nnz;

    // the part's first row: max { i in [0, rows] : pos[i] <= b0 }; every thread runs the same search
    int r0;
    {
        int lo = 0, hi = rows;
        while (lo < hi) {
            const int mid = lo + ((hi - lo + 1) >> 1);
            if (pos[mid] <= b0) lo = mid; else hi = mid - 1;
        }
        r0 = lo;
    }
    const int part_r0 = r0;
    const bool part_carry = (p > 0) && (pos[r0] < b0);
    if (tid == 0) {
        if (!part_carry) carry_row[p] = -1;
        s_pend[0] = 0.0f;
        s_pend[1] = 0.0f;
    }

    // The chunks are counted, not stepped by position: near nnz = 2^31 - 1 a position that is advanced past
    // the end of the part would wrap around.  b0 + c*T < b1 <= nnz for every chunk c of the part.
    const int nchunks = (int)(((long long)b1 - b0 + T - 1) / T);
    int parity = 0;
    for (int c = 0; c < nchunks; ++c, parity ^= 1) {
        const int t0 = b0 + c * T;
        const int cnt = (b1 - t0 < T) ? b1 - t0 : T;
        const int t1 = t0 + cnt;
        const bool last = t1 == b1;

        // ---- stream + gather + multiply (the per-thread temporary and the unrolled load loop)
        float prod[NPT];
        if (cnt == T) {
            if (VEC) {
                v4i cv[NPT / 4];
                v4f vv[NPT / 4];
#pragma unroll
                for (int g = 0; g < NPT / 4; ++g) {
                    const int off = t0 + (g * THREADS + tid) * 4;
                    cv[g] = ld_stream(reinterpret_cast<const v4i *>(crd + off));
                    vv[g] = ld_stream(reinterpret_cast<const v4f *>(vals + off));
                }
                // two 16-byte gathers per four positions when every lane of the wave holds two runs of consecutive
                // columns (run_plan), four 4-byte gathers otherwise: as in the tiled kernel
                float xg[NPT / 4][4];
                RunPlan plan[NPT / 4];
                bool ok = true;
#pragma unroll
                for (int g = 0; g < NPT / 4; ++g) {
                    plan[g] = run_plan(cv[g], cols);
                    ok = ok && plan[g].ok;
                }
                if (__ballot(!ok) == 0ull) {
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
                        xg[g][0] = x[cv[g].x]; xg[g][1] = x[cv[g].y]; xg[g][2] = x[cv[g].z]; xg[g][3] = x[cv[g].w];
                    }
                }
#pragma unroll
                for (int g = 0; g < NPT / 4; ++g) {
                    prod[4 * g] = vv[g].x * xg[g][0];
                    prod[4 * g + 1] = vv[g].y * xg[g][1];
                    prod[4 * g + 2] = vv[g].z * xg[g][2];
                    prod[4 * g + 3] = vv[g].w * xg[g][3];
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
        } else {
#pragma unroll
            for (int g = 0; g < NPT; ++g) {
                const int i = VEC ? ((g / 4) * THREADS + tid) * 4 + (g & 3) : g * THREADS + tid;
                prod[g] = i < cnt ? vals[t0 + i] * x[crd[t0 + i]] : 0.0f;
            }
        }
        if (tid == 0) { nlong = 0; s_next = r0; s_pend[parity ^ 1] = 0.0f; }
#pragma unroll
        for (int g = 0; g < NPT; ++g) {
            const int i = VEC ? ((g / 4) * THREADS + tid) * 4 + (g & 3) : g * THREADS + tid;
            sprod[skew<1>(i)] = prod[g];
        }
        __syncthreads();
        const float pend_in = s_pend[parity];

        // A finished row segment.  before: the row began before this chunk (only the chunk's first row
        // can); after: it goes on past the chunk (only its last row can).
        auto finish = [&](int r, float s, bool before, bool after) {
            const float total = before ? pend_in + s : s;
            if (after && !last) {
                s_pend[parity ^ 1] = total;                     // continues in the next chunk of this part
            } else if (part_carry && r == part_r0) {
                carry_row[p] = r;                               // began in an earlier part
                carry_val[p] = total;
            } else {
                y[r] = total;                                   // complete, or this part owns its head
            }
        };

        // ---- rows of the chunk, THREADS at a time, until one lies beyond it
        const int rbeg = (t0 == 0) ? 0 : r0;
        for (int rb = rbeg;; rb += THREADS) {
            const int r = rb + tid;
            const int a = pos[r < rows ? r : rows], b = pos[r + 1 < rows ? r + 1 : rows];
            if (r <= rows && a <= t1) atomicMax(&s_next, r);
            const bool mine = r < rows && (a < t1 || b <= t1);
            if (mine) {
                int lo = a - t0, hi = b - t0;
                const bool before = lo < 0, after = hi > cnt;
                lo = before ? 0 : lo;
                hi = after ? cnt : hi;
                if (hi - lo < LONG) {
                    float s = 0.0f;
                    int i = lo;
                    for (; i + 4 <= hi; i += 4) {
                        const float q0 = sprod[skew<1>(i)], q1 = sprod[skew<1>(i + 1)], q2 = sprod[skew<1>(i + 2)],
                                    q3 = sprod[skew<1>(i + 3)];
                        s += q0; s += q1; s += q2; s += q3;
                    }
                    for (; i < hi; ++i) s += sprod[skew<1>(i)];
                    finish(r, s, before, after);
                } else {
                    const int e = atomicAdd(&nlong, 1);
                    if (e < MAXLONG) {
                        slong[4 * e] = r; slong[4 * e + 1] = lo; slong[4 * e + 2] = hi;
                        slong[4 * e + 3] = (before ? 1 : 0) | (after ? 2 : 0);
                    }
                }
            }
            if (__syncthreads_count(mine) != THREADS) break;   // uniform: the count is the same in every thread
        }
        const int nl = nlong < MAXLONG ? nlong : MAXLONG;
        for (int e = wave; e < nl; e += NW) {
            const int r = slong[4 * e], lo = slong[4 * e + 1], hi = slong[4 * e + 2], fl = slong[4 * e + 3];
            float s = 0.0f;
            for (int i = lo + lane; i < hi; i += WAVE) s += sprod[skew<1>(i)];
            s = wave_sum(s);
            if (lane == 0) finish(r, s, (fl & 1) != 0, (fl & 2) != 0);
        }
        r0 = s_next;
        __syncthreads();                                        // sprod, nlong, s_next are reused
    }
}

hipError_t launch_spmv_csr_divide(int32_t rows, int32_t cols, int32_t nnz, const int32_t *pos, const int32_t *crd,
                                  const float *vals, const float *x, float *y, int32_t parts,
                                  int32_t chunks_per_part, const Workspace &w, hipStream_t s)
{
    if (parts <= 0) return hipSuccess;
    const bool vec = ((reinterpret_cast<uintptr_t>(crd) | reinterpret_cast<uintptr_t>(vals)) & 15) == 0;
    if (vec)
        PSK_LAUNCH((k_spmv_div<256, 8, true>), dim3(parts), dim3(256), 0, s, rows, cols, nnz, pos, crd, vals, x, y,
                           w.carry_row, w.carry_val, chunks_per_part);
    else
        PSK_LAUNCH((k_spmv_div<256, 8, false>), dim3(parts), dim3(256), 0, s, rows, cols, nnz, pos, crd, vals, x, y,
                           w.carry_row, w.carry_val, chunks_per_part);
    return take_launch_status();
}

}  // namespace psk
