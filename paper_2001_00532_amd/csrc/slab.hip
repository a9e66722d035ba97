// Column-slab hierarchy of a CSR matrix: the analysis step that builds it and the first step of the
// SpMV over it.
//
// Why: on this chip a 4-byte gather of x that misses the 32 KB L1 costs one 64-byte request slot of the
// L1's miss path whatever the table's size, and a row-ordered CSR with scattered columns misses almost
// always.  Section 8.6 of the paper gets locality by tiling (split a loop, move the outer part outward);
// Section 3 lets the position cut be taken in any coordinate hierarchy.  Here the column loop j is split
// by a slab of PSK_SLAB_COLS columns, jo = j / PSK_SLAB_COLS moves outermost and A is STORED in that
// order once (three levels: jo dense, i compressed, ji compressed).  The position space of the leaf
// level is then cut into equal pieces as before, but a piece now needs only one slab of x, which a
// workgroup keeps in on-chip memory (128 KB of the CU's 160 KB): gathers become LDS reads.
//
// Structure (all built here, on the device; the CPU oracle builds the same arrays from the definition):
//   slots   = the stored entries sorted by (slab, CSR position): a stable bucketing; every slab is
//             padded to a multiple of PSK_SLAB_CHUNK slots so that a chunk never crosses a slab;
//   pair    = a maximal run of slots of one row inside one chunk; scol bit 15 marks a pair's last slot;
//   step 1  : P[pair] = sum of value * x over the pair's slots            (k_slab_pairs, this file)
//   step 2  : y[i] = sum of P over the pairs of row i, listed by (qpos, qidx): the ordinary position-cut
//             SpMV kernel with unit values (k_spmv_pos, VARIANT 6).
// A chunk is one wave's unit of work: no sum crosses a chunk, so step 1 needs no communication between
// waves, no carries and no barrier except when a workgroup moves on to the next slab.
#include "psk_dev.h"
#include "psk_internal.h"

namespace psk {

constexpr int SLAB_CH = kSlabChunk;
constexpr int BUILD_BT = kSlabBuildBlock;     // CSR positions per block of the bucketing kernels

// Per value type: columns per slab (what fits into the LDS next to the staging area) and values per 16 bytes.
typedef double v2d __attribute__((ext_vector_type(2)));
template <typename T> struct SlabOf;
template <> struct SlabOf<float>  { static constexpr int W = kSlabCols,    G = 4, WAVES = 16; typedef v4f V; };
template <> struct SlabOf<double> { static constexpr int W = kSlabColsF64, G = 2, WAVES = kSlabWavesF64; typedef v2d V; };

// Where the value of slot j is stored.  A lane of the pair kernel owns 8 consecutive slots of a chunk; stored in
// slot order its 16-byte loads would each touch every other 16 bytes of the chunk.  Inside each chunk the values
// are therefore stored in groups of G = 16 bytes / value size: [first G slots of lane 0, of lane 1, ... | next G
// slots of lane 0, ...], so that every load is contiguous over the wave (measured for fp32 on the streams alone: 60
// instead of 65 us).
template <int G>
__host__ __device__ __forceinline__ int slab_value_index(int j)
{
    const int o = j & (SLAB_CH - 1), l = o >> 3, k = o & 7;
    return (j - o) + (k / G) * (SLAB_CH / 8 * G) + G * l + (k % G);
}

// ------------------------------------------------------------------ DPP scans over the 64 lanes of a wave
template <int CTRL, int ROWMASK>
__device__ __forceinline__ int dpp_i(int v) { return __builtin_amdgcn_update_dpp(0, v, CTRL, ROWMASK, 0xF, false); }
template <int CTRL, int ROWMASK>
__device__ __forceinline__ float dpp_f(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROWMASK, 0xF, false));
}
template <int CTRL, int ROWMASK>
__device__ __forceinline__ double dpp_f(double v)
{
    const long long b = __builtin_bit_cast(long long, v);
    const unsigned lo = (unsigned)dpp_i<CTRL, ROWMASK>((int)(unsigned)b), hi = (unsigned)dpp_i<CTRL, ROWMASK>((int)(b >> 32));
    return __builtin_bit_cast(double, (long long)(((unsigned long long)hi << 32) | lo));
}
// row_shr 1, 2, 4, 8 scan each row of 16 lanes; row_bcast15 hands lane 15 of rows 0 and 2 to rows 1 and 3,
// row_bcast31 hands lane 31 to rows 2 and 3.  Lanes without a source receive 0.
__device__ __forceinline__ int wave_scan_add(int v)
{
    v += dpp_i<0x111, 0xF>(v);
    v += dpp_i<0x112, 0xF>(v);
    v += dpp_i<0x114, 0xF>(v);
    v += dpp_i<0x118, 0xF>(v);
    v += dpp_i<0x142, 0xA>(v);
    v += dpp_i<0x143, 0xC>(v);
    return v;
}
// Inclusive segmented sum: a lane with f != 0 starts afresh (takes nothing from the lanes below it).
template <typename T>
__device__ __forceinline__ T wave_segscan(T v, int f)
{
#define PSK_SEG_STEP(CTRL, MASK)                       \
    {                                                  \
        const T pv = dpp_f<CTRL, MASK>(v);             \
        const int pf = dpp_i<CTRL, MASK>(f);           \
        v = f ? v : v + pv;                            \
        f |= pf;                                       \
    }
    PSK_SEG_STEP(0x111, 0xF) PSK_SEG_STEP(0x112, 0xF) PSK_SEG_STEP(0x114, 0xF) PSK_SEG_STEP(0x118, 0xF)
    PSK_SEG_STEP(0x142, 0xA) PSK_SEG_STEP(0x143, 0xC)
#undef PSK_SEG_STEP
    return v;
}

// ------------------------------------------------------------------ step 1 of the product
// Persistent workgroups: every workgroup owns one piece of cpw consecutive chunks (the position space DIVIDED into
// equal pieces, Section 5), walks them slab by slab, loads the slab's part of x into LDS once and lets its
// waves (16; 8 for fp64) take the chunks of that slab round-robin.  A lane owns 8 consecutive slots (two 16-byte loads of
// values, one of columns); the next chunk's loads are issued before the current one is processed.
// Inside a chunk (no branches): the lane walks its 8 slots with a running sum that restarts after a pair
// end and writes every running sum to LDS -- to the pair's place in the chunk (number of pair ends before
// it) when the slot ends a pair, to a dummy word otherwise; a segmented DPP scan then hands each lane the
// open sum of the lanes below it, which is added to the lane's first pair.  The chunk's pair sums, now
// compact in LDS, leave with full-width coalesced stores to P[chunk_pair[c] ...].
// LDS: 127.9 KB of x + 2 KB of pair sums per wave + the dummy words = the CU's 160 KB (fp64: 8 waves, 127.75 KB of
// x = 16 352 columns, + 4 KB of pair sums per wave; 16 waves with 12 256 columns measured the same, 191.5 against
// 190.3 us on the power-law configuration, and make more pairs).
template <typename T>
__global__ __launch_bounds__(SlabOf<T>::WAVES * WAVE) void k_slab_pairs(const T *__restrict__ svals,
                                                     const unsigned short *__restrict__ scol,
                                                     const int *__restrict__ chunk_pair,
                                                     const int *__restrict__ slab_chunk,
                                                     const T *__restrict__ x, T *__restrict__ P, int cols,
                                                     int nslabs, int nchunks, int cpw, int *__restrict__ gap)
{
    constexpr int WAVES = SlabOf<T>::WAVES;
    constexpr int W = SlabOf<T>::W, G = SlabOf<T>::G, NV = 8 / G;      // NV 16-byte loads of values per lane
    typedef typename SlabOf<T>::V V;
    // the run list of the second step starts empty (that step's tiles append to it, the fix-up consumes it)
    if (blockIdx.x == 0 && threadIdx.x == 0 && gap) { gap[0] = 0; gap[1] = 0; }
    __shared__ T xs[W];
    __shared__ T stage[WAVES * SLAB_CH + 32];         // + one dummy word per LDS bank
    static_assert(sizeof(T) * (W + WAVES * SLAB_CH + 32) <= 163840, "the window and the staging area fill the CU's LDS");
    const int tid = threadIdx.x, lane = tid & (WAVE - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / WAVE);
    T *st = stage + wave * SLAB_CH;
    const int dummy = (WAVES - wave) * SLAB_CH + (lane & 31);      // index, relative to st, of a word nobody reads
    // piece of this workgroup: neighbouring pieces go to workgroups of the same die, so that the slabs of x they share
    // are fetched into that die's L2 once (measured on the power-law matrix: 76.2 against 79.4 us)
    const int piece = xcd_tile(blockIdx.x, (nchunks + cpw - 1) / cpw);
    if (piece < 0) return;
    int c0 = piece * cpw;
    const int c1 = min(c0 + cpw, nchunks);
    if (c0 >= c1) return;
    PSK_TRACE_WORKGROUP();
    int s;      // slab of chunk c0: max { s : slab_chunk[s] <= c0 }
    {
        int lo = 0, hi = nslabs;
        while (lo < hi) {
            const int mid = lo + ((hi - lo + 1) >> 1);
            if (slab_chunk[mid] <= c0) lo = mid; else hi = mid - 1;
        }
        s = lo;
    }
    while (c0 < c1) {
        while (slab_chunk[s + 1] <= c0) ++s;            // skips empty slabs; c0 < nchunks = slab_chunk[nslabs]
        const int ce = min(c1, slab_chunk[s + 1]);
        __syncthreads();                                  // the previous slab's window is no longer read
        const long long xb = (long long)s * W;
        const int wlen = (int)min((long long)W, (long long)cols - xb);
        const bool x16 = (reinterpret_cast<uintptr_t>(x + xb) & 15) == 0;
        for (int i = tid * G; i < wlen; i += WAVES * WAVE * G) {
            if (x16 && i + G <= wlen) {
                *reinterpret_cast<V *>(&xs[i]) = *reinterpret_cast<const V *>(x + xb + i);
            } else {
                for (int j = i; j < i + G && j < wlen; ++j) xs[j] = x[xb + j];
            }
        }
        __syncthreads();
        int c = c0 + wave;
        V va[NV];
#pragma unroll
        for (int g = 0; g < NV; ++g) va[g] = V{};
        v4i cc = {0, 0, 0, 0};
        int pb = 0;
        auto issue = [&](int ci) {
            const long long b = (long long)ci * SLAB_CH;
#pragma unroll
            for (int g = 0; g < NV; ++g)                                       // slots 8*lane + g*G .. + G-1
                va[g] = ld_stream(reinterpret_cast<const V *>(svals + b + g * (SLAB_CH / 8 * G) + lane * G));
            cc = ld_stream(reinterpret_cast<const v4i *>(scol + b + lane * 8));
            // lanes 0 and 1 fetch the chunk's first pair and the next chunk's: a vector load on purpose, a scalar
            // load would share its counter with the LDS reads and make each of them wait for its round trip
            pb = chunk_pair[ci + (lane & 1)];
        };
        if (c < ce) issue(c);
        for (; c < ce; c += WAVES) {
            T v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = va[j / G][j % G];
            const v4i q = cc;
            const int pbase = rl(pb, 0), np = rl(pb, 1) - pbase;
            if (c + WAVES < ce) issue(c + WAVES);
            const unsigned w0 = (unsigned)q.x, w1 = (unsigned)q.y, w2 = (unsigned)q.z, w3 = (unsigned)q.w;
            // bit j = slot j of this lane ends a pair (bit 15 of its 16-bit column word)
            const unsigned ends = ((w0 >> 15) & 1u) | ((w0 >> 30) & 2u) | ((w1 >> 13) & 4u) | ((w1 >> 28) & 8u) |
                                  ((w2 >> 11) & 16u) | ((w2 >> 26) & 32u) | ((w3 >> 9) & 64u) | ((w3 >> 24) & 128u);
            const unsigned w[4] = {w0, w1, w2, w3};
            T p[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const unsigned h = (j & 1) ? (w[j >> 1] >> 16) : w[j >> 1];
                p[j] = v[j] * xs[h & 0x7fffu];
            }
            const int cnt = __popc(ends);
            const int first = wave_scan_add(cnt) - cnt;         // place of this lane's first pair end in the chunk
            T run = 0;
            int place = first;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const bool e = (ends >> j) & 1u;
                run += p[j];
                st[e ? place : dummy] = run;
                run = e ? T(0) : run;
                place += e ? 1 : 0;
            }
            // `run` is the lane's open sum; the lane below hands over the open sum of all lanes below it
            const T open = wave_segscan<T>(run, cnt ? 1 : 0);
            const T carry = __shfl_up(open, 1, WAVE);
            if (cnt && lane) st[first] += carry;                // head + carry (a chunk's first slot starts a pair)
            for (int k = lane; k < np; k += WAVE) P[pbase + k] = st[k];
        }
        c0 = ce;
        ++s;
    }
}

template <typename T>
static hipError_t launch_slab_pairs_t(const T *svals, const uint16_t *scol, const int32_t *chunk_pair,
                                      const int32_t *slab_chunk, const T *x, T *P, int32_t cols, int32_t nslabs,
                                      int32_t nchunks, int32_t nwg, int32_t *gap, hipStream_t s)
{
    if (nchunks <= 0) return hipSuccess;
    if (nwg < 1) nwg = 1;
    const int cpw = (nchunks + nwg - 1) / nwg;
    const int grid = xcd_grid((nchunks + cpw - 1) / cpw);
    PSK_LAUNCH(k_slab_pairs<T>, dim3(grid), dim3(SlabOf<T>::WAVES * WAVE), 0, s, svals, scol, chunk_pair, slab_chunk, x, P, cols, nslabs,
               nchunks, cpw, gap);
    return take_launch_status();
}

hipError_t launch_slab_pairs(const float *svals, const uint16_t *scol, const int32_t *chunk_pair,
                             const int32_t *slab_chunk, const float *x, float *P, int32_t cols, int32_t nslabs,
                             int32_t nchunks, int32_t nwg, int32_t *gap, hipStream_t s)
{
    return launch_slab_pairs_t<float>(svals, scol, chunk_pair, slab_chunk, x, P, cols, nslabs, nchunks, nwg, gap, s);
}

hipError_t launch_slab_pairs_f64(const double *svals, const uint16_t *scol, const int32_t *chunk_pair,
                                 const int32_t *slab_chunk, const double *x, double *P, int32_t cols, int32_t nslabs,
                                 int32_t nchunks, int32_t nwg, int32_t *gap, hipStream_t s)
{
    return launch_slab_pairs_t<double>(svals, scol, chunk_pair, slab_chunk, x, P, cols, nslabs, nchunks, nwg, gap, s);
}

// ------------------------------------------------------------------ prefix sums over int32 arrays
// Exclusive scans.  Three kernels: sums of blocks of 4096, a single-workgroup scan of those sums, then every block
// scans its own elements on top of its offset.  In place (out == in) is allowed.
constexpr int SCAN_EPT = 16, SCAN_BLOCK = 256 * SCAN_EPT;

__device__ __forceinline__ int block_scan_256(int v, int *s_w, int *total)
{
    // inclusive scan of one value per thread over 256 threads; s_w has 4 ints
    const int lane = threadIdx.x & (WAVE - 1), wave = threadIdx.x / WAVE;
    const int inc = wave_scan_add(v);
    if (lane == WAVE - 1) s_w[wave] = inc;
    __syncthreads();
    int off = 0;
    for (int w = 0; w < wave; ++w) off += s_w[w];
    *total = s_w[0] + s_w[1] + s_w[2] + s_w[3];
    __syncthreads();
    return inc + off;
}

// a thread's SCAN_EPT consecutive elements, as four 16-byte loads when they all exist (the arrays start on 256-byte
// boundaries and a thread's share on a 64-byte one)
template <bool NONZERO>
__device__ __forceinline__ void scan_load(const int *__restrict__ in, long long base, long long n, int (&v)[SCAN_EPT])
{
    if (base + SCAN_EPT <= n) {
#pragma unroll
        for (int g = 0; g < SCAN_EPT / 4; ++g) {
            const v4i t = *reinterpret_cast<const v4i *>(in + base + 4 * g);
            v[4 * g] = t.x; v[4 * g + 1] = t.y; v[4 * g + 2] = t.z; v[4 * g + 3] = t.w;
        }
    } else {
#pragma unroll
        for (int i = 0; i < SCAN_EPT; ++i) v[i] = base + i < n ? in[base + i] : 0;
    }
    if (NONZERO) {
#pragma unroll
        for (int i = 0; i < SCAN_EPT; ++i) v[i] = v[i] != 0;
    }
}

// NONZERO: the scanned sequence is (in[i] != 0)
template <bool NONZERO>
__global__ __launch_bounds__(256) void k_scan_reduce(const int *__restrict__ in, long long n, int *__restrict__ bsum)
{
    __shared__ int s_w[4];
    const long long base = (long long)blockIdx.x * SCAN_BLOCK + threadIdx.x * SCAN_EPT;
    int v[SCAN_EPT];
    scan_load<NONZERO>(in, base, n, v);
    int t = 0;
#pragma unroll
    for (int i = 0; i < SCAN_EPT; ++i) t += v[i];
    int total;
    block_scan_256(t, s_w, &total);
    if (threadIdx.x == 0) bsum[blockIdx.x] = total;
}

// exclusive scan of bsum[0 .. nb) in place, by one workgroup of 256 threads
__global__ __launch_bounds__(256) void k_scan_spine(int *__restrict__ bsum, long long nb)
{
    __shared__ int s_w[4];
    int carry = 0;
    for (long long b0 = 0; b0 < nb; b0 += 256) {
        const long long i = b0 + threadIdx.x;
        const int v = i < nb ? bsum[i] : 0;
        int total;
        const int inc = block_scan_256(v, s_w, &total);
        if (i < nb) bsum[i] = carry + inc - v;
        carry += total;
    }
}

template <bool NONZERO>
__global__ __launch_bounds__(256) void k_scan_apply(const int *__restrict__ in, int *__restrict__ out, long long n,
                                                    const int *__restrict__ bsum)
{
    __shared__ int s_w[4];
    const long long base = (long long)blockIdx.x * SCAN_BLOCK + threadIdx.x * SCAN_EPT;
    int v[SCAN_EPT];
    scan_load<NONZERO>(in, base, n, v);
    int t = 0;
#pragma unroll
    for (int i = 0; i < SCAN_EPT; ++i) t += v[i];
    int total;
    const int inc = block_scan_256(t, s_w, &total);
    int run = bsum[blockIdx.x] + inc - t;
    int o[SCAN_EPT];
#pragma unroll
    for (int i = 0; i < SCAN_EPT; ++i) {
        o[i] = run;
        run += v[i];
    }
    if (base + SCAN_EPT <= n) {
#pragma unroll
        for (int g = 0; g < SCAN_EPT / 4; ++g)
            *reinterpret_cast<v4i *>(out + base + 4 * g) = v4i{o[4 * g], o[4 * g + 1], o[4 * g + 2], o[4 * g + 3]};
    } else {
#pragma unroll
        for (int i = 0; i < SCAN_EPT; ++i)
            if (base + i < n) out[base + i] = o[i];
    }
}

size_t scan_tmp_ints(int64_t n) { return (size_t)((n + SCAN_BLOCK - 1) / SCAN_BLOCK) + 1; }

// exclusive scan of in[0 .. n) into out (in place allowed); nonzero: of the sequence (in[i] != 0)
static void launch_scan(const int32_t *in, int32_t *out, int64_t n, int32_t *bsum, bool nonzero, hipStream_t s)
{
    if (n <= 0) return;
    const long long nb = (n + SCAN_BLOCK - 1) / SCAN_BLOCK;
    if (nonzero) PSK_LAUNCH(k_scan_reduce<true>, dim3((unsigned)nb), dim3(256), 0, s, in, (long long)n, bsum);
    else PSK_LAUNCH(k_scan_reduce<false>, dim3((unsigned)nb), dim3(256), 0, s, in, (long long)n, bsum);
    PSK_LAUNCH(k_scan_spine, dim3(1), dim3(256), 0, s, bsum, nb);
    if (nonzero) PSK_LAUNCH(k_scan_apply<true>, dim3((unsigned)nb), dim3(256), 0, s, in, out, (long long)n, bsum);
    else PSK_LAUNCH(k_scan_apply<false>, dim3((unsigned)nb), dim3(256), 0, s, in, out, (long long)n, bsum);
}

// ------------------------------------------------------------------ the analysis step: CSR -> slab hierarchy
// H[s * nblk + b] = number of positions of block b (BUILD_BT consecutive CSR positions) that fall into slab s.
__global__ __launch_bounds__(256) void k_slab_hist(int nnz, const int *__restrict__ crd, int W, int nslabs, int nblk,
                                                   int *__restrict__ H)
{
    extern __shared__ int hist[];
    for (int s = threadIdx.x; s < nslabs; s += 256) hist[s] = 0;
    __syncthreads();
    const int b = blockIdx.x;
    const long long p0 = (long long)b * BUILD_BT;
    for (int i = threadIdx.x; i < BUILD_BT; i += 256)
        if (p0 + i < nnz) atomicAdd(&hist[crd[p0 + i] / W], 1);
    __syncthreads();
    for (int s = threadIdx.x; s < nslabs; s += 256) H[(long long)s * nblk + b] = hist[s];
}

// E = exclusive scan of H (E[nslabs * nblk] = nnz).  One workgroup: slab s holds E[(s+1)*nblk] - E[s*nblk]
// positions, padded to a multiple of the chunk; slab_chunk = exclusive scan of the padded sizes in chunks.
// meta[0] = number of slots.
__global__ __launch_bounds__(256) void k_slab_bases(const int *__restrict__ E, int nslabs, int nblk,
                                                    int *__restrict__ slab_chunk, int *__restrict__ meta)
{
    __shared__ int s_w[4];
    int carry = 0;
    for (int s0 = 0; s0 < nslabs; s0 += 256) {
        const int s = s0 + threadIdx.x;
        int chunks = 0;
        if (s < nslabs) {
            const int cnt = E[(long long)(s + 1) * nblk] - E[(long long)s * nblk];
            chunks = (cnt + SLAB_CH - 1) / SLAB_CH;
        }
        int total;
        const int inc = block_scan_256(chunks, s_w, &total);
        if (s < nslabs) slab_chunk[s] = carry + inc - chunks;
        carry += total;
    }
    if (threadIdx.x == 0) {
        slab_chunk[nslabs] = carry;
        meta[0] = carry * SLAB_CH;
    }
}

// The pad slots of slab s (fewer than a chunk): value 0, column 0, no row, no source position.
template <typename T>
__global__ __launch_bounds__(64) void k_slab_pads(const int *__restrict__ E, int nblk, const int *__restrict__ slab_chunk,
                                                  T *__restrict__ svals, unsigned short *__restrict__ scol,
                                                  int *__restrict__ srow, int *__restrict__ src)
{
    const int s = blockIdx.x;
    const int cnt = E[(long long)(s + 1) * nblk] - E[(long long)s * nblk];
    const long long lo = (long long)slab_chunk[s] * SLAB_CH + cnt, hi = (long long)slab_chunk[s + 1] * SLAB_CH;
    for (long long j = lo + threadIdx.x; j < hi; j += 64) {
        svals[slab_value_index<SlabOf<T>::G>((int)j)] = T(0);
        scol[j] = 0;
        srow[j] = -1;
        src[j] = -1;
    }
}

// Stable bucketing.  One wave per block of BUILD_BT CSR positions, taken 64 at a time in order; off[s] is the
// slot the block's next position of slab s goes to.  The lanes of one step that share a slab are ranked by
// lane number, so the order of the CSR is kept inside every slab: `nbits` ballots, one per bit of the slab
// number, leave every lane with the mask of the lanes of its slab.  The row of a position is the largest r
// with pos[r] <= p, searched between the rows of the block's first and last position (tile_row = the position
// cut of pos with tiles of BUILD_BT) -- in a copy of that part of pos in LDS when it has at most SCATTER_ROWS
// entries, in global memory otherwise.  The loads of the next 64 positions are issued before the current ones
// are placed.
constexpr int SCATTER_ROWS = 1024;
template <typename T>
__global__ __launch_bounds__(64) void k_slab_scatter(int rows, int nnz, const int *__restrict__ pos,
                                                     const int *__restrict__ crd, const T *__restrict__ vals,
                                                     const int *__restrict__ tile_row, const int *__restrict__ E,
                                                     const int *__restrict__ slab_chunk, int nslabs, int nblk,
                                                     int nbits, T *__restrict__ svals,
                                                     unsigned short *__restrict__ scol, int *__restrict__ srow,
                                                     int *__restrict__ src)
{
    extern __shared__ int off[];                 // [nslabs] next slot of each slab, then [SCATTER_ROWS] row starts
    constexpr int W = SlabOf<T>::W;
    const int b = blockIdx.x, lane = threadIdx.x;
    int *spos = off + nslabs;
    for (int s = lane; s < nslabs; s += WAVE)
        off[s] = slab_chunk[s] * SLAB_CH + (E[(long long)s * nblk + b] - E[(long long)s * nblk]);
    const long long p0 = (long long)b * BUILD_BT;
    const int r_lo = tile_row[b], r_hi = tile_row[b + 1];
    const bool local = r_hi - r_lo < SCATTER_ROWS;          // rows r_lo .. r_hi: at most SCATTER_ROWS of them
    if (local)
        for (int i = lane; i <= r_hi - r_lo; i += WAVE) spos[i] = pos[r_lo + i];
    __syncthreads();
    const unsigned long long below = (1ull << lane) - 1ull;
    int c_next = 0;
    T v_next = 0;
    if (p0 + lane < nnz) { c_next = crd[p0 + lane]; v_next = vals[p0 + lane]; }
    for (int it = 0; it < BUILD_BT / WAVE; ++it) {
        const long long pl = p0 + it * WAVE + lane;
        const bool valid = pl < nnz;
        const int p = valid ? (int)pl : 0;
        const int c = c_next;
        const T v = v_next;
        if (it + 1 < BUILD_BT / WAVE && pl + WAVE < nnz) { c_next = crd[pl + WAVE]; v_next = vals[pl + WAVE]; }
        const int s = valid ? c / W : 0;
        int r = 0;
        if (valid) {
            int lo = r_lo, hi = r_hi;
            if (local) {
                while (lo < hi) {
                    const int mid = lo + ((hi - lo + 1) >> 1);
                    if (spos[mid - r_lo] <= p) lo = mid; else hi = mid - 1;
                }
            } else {
                while (lo < hi) {
                    const int mid = lo + ((hi - lo + 1) >> 1);
                    if (pos[mid] <= p) lo = mid; else hi = mid - 1;
                }
            }
            r = lo;
        }
        // peers = the valid lanes with the same slab number
        unsigned long long peers = __ballot(valid);
        for (int k = 0; k < nbits; ++k) {
            const bool one = (s >> k) & 1;
            const unsigned long long m = __ballot(valid && one);
            peers &= one ? m : ~m;
        }
        int dst = -1;
        if (valid) dst = off[s] + __popcll(peers & below);
        __syncthreads();                                  // one wave: orders the LDS reads before the updates
        if (valid && (peers & below) == 0) off[s] += __popcll(peers);
        __syncthreads();
        if (valid) {
            svals[slab_value_index<SlabOf<T>::G>(dst)] = v;
            scol[dst] = (unsigned short)(c - s * W);
            srow[dst] = r;
            src[dst] = p;
        }
    }
}

// The same bucketing for matrices of at most STAGE_SLABS slabs, with coalesced stores: a workgroup of four waves takes
// the block, wave w its w-th quarter (8 steps of 64 positions).  The waves first count their positions per slab; from
// the counts every (wave, slab) gets its place in a staging area in LDS that holds the block's entries ordered by slab
// (and inside a slab by CSR position: wave after wave, step after step, lane after lane -- the same stable order).  The
// entries are then ranked as above, staged, and written out in staging order, so that a slab's entries of this block
// (33 on average for 62 slabs) leave as one run of consecutive slots instead of 64 scattered stores per step.
constexpr int STAGE_SLABS = 256;
template <typename T>
__global__ __launch_bounds__(256) void k_slab_scatter_staged(int rows, int nnz, const int *__restrict__ pos,
                                                            const int *__restrict__ crd, const T *__restrict__ vals,
                                                            const int *__restrict__ tile_row,
                                                            const int *__restrict__ E,
                                                            const int *__restrict__ slab_chunk, int nslabs, int nblk,
                                                            int nbits, T *__restrict__ svals,
                                                            unsigned short *__restrict__ scol,
                                                            int *__restrict__ srow, int *__restrict__ src)
{
    constexpr int W = SlabOf<T>::W, NW = 4, QUART = BUILD_BT / NW, STEPS = QUART / WAVE;
    __shared__ int woff[NW][STAGE_SLABS];        // entries of (wave, slab); later: where that wave's next entry of the slab goes
    __shared__ int lbase[STAGE_SLABS + 1];       // first staging index of each slab
    __shared__ int gbase[STAGE_SLABS];           // first slot (global) of this block's entries of each slab
    __shared__ int spos[SCATTER_ROWS];
    __shared__ T s_val[BUILD_BT];
    __shared__ int s_row[BUILD_BT];
    __shared__ unsigned short s_col[BUILD_BT], s_idx[BUILD_BT], s_slab[BUILD_BT];
    __shared__ int s_w[4];
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & (WAVE - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / WAVE);
    const long long p0 = (long long)b * BUILD_BT;
    const int nvalid = (int)min((long long)BUILD_BT, (long long)nnz - p0);
    const int r_lo = tile_row[b], r_hi = tile_row[b + 1];
    const bool local = r_hi - r_lo < SCATTER_ROWS;
    for (int i = tid; i < NW * STAGE_SLABS; i += 256) (&woff[0][0])[i] = 0;
    if (local)
        for (int i = tid; i <= r_hi - r_lo; i += 256) spos[i] = pos[r_lo + i];
    for (int sl = tid; sl < nslabs; sl += 256)
        gbase[sl] = slab_chunk[sl] * SLAB_CH + (E[(long long)sl * nblk + b] - E[(long long)sl * nblk]);
    __syncthreads();
    // this lane's positions: wave * QUART + st * 64 + lane
    int c[STEPS], r[STEPS];
    T v[STEPS];
#pragma unroll
    for (int st = 0; st < STEPS; ++st) {
        const int i = wave * QUART + st * WAVE + lane;
        c[st] = 0; v[st] = T(0);
        if (i < nvalid) { c[st] = crd[p0 + i]; v[st] = vals[p0 + i]; }
    }
#pragma unroll
    for (int st = 0; st < STEPS; ++st) {
        const int i = wave * QUART + st * WAVE + lane;
        r[st] = 0;
        if (i < nvalid) {
            const int p = (int)(p0 + i);
            atomicAdd(&woff[wave][c[st] / W], 1);
            int lo = r_lo, hi = r_hi;
            if (local) {
                while (lo < hi) {
                    const int mid = lo + ((hi - lo + 1) >> 1);
                    if (spos[mid - r_lo] <= p) lo = mid; else hi = mid - 1;
                }
            } else {
                while (lo < hi) {
                    const int mid = lo + ((hi - lo + 1) >> 1);
                    if (pos[mid] <= p) lo = mid; else hi = mid - 1;
                }
            }
            r[st] = lo;
        }
    }
    __syncthreads();
    // staging index of each slab = exclusive scan of the block's count per slab (two slabs per thread), then the
    // waves' places inside each slab
    {
        const int s0 = 2 * tid, s1 = 2 * tid + 1;
        int n0 = 0, n1 = 0;
        if (s0 < nslabs) n0 = woff[0][s0] + woff[1][s0] + woff[2][s0] + woff[3][s0];
        if (s1 < nslabs) n1 = woff[0][s1] + woff[1][s1] + woff[2][s1] + woff[3][s1];
        int total;
        const int inc = block_scan_256(n0 + n1, s_w, &total);
        const int b0 = inc - n0 - n1;
        if (s0 < nslabs) {
            lbase[s0] = b0;
            int o = b0;
            for (int w = 0; w < NW; ++w) { const int t = woff[w][s0]; woff[w][s0] = o; o += t; }
        }
        if (s1 < nslabs) {
            lbase[s1] = b0 + n0;
            int o = b0 + n0;
            for (int w = 0; w < NW; ++w) { const int t = woff[w][s1]; woff[w][s1] = o; o += t; }
        }
    }
    __syncthreads();
    // rank and stage (a wave touches only its own row of woff; its LDS operations execute in program order)
    const unsigned long long below = (1ull << lane) - 1ull;
#pragma unroll
    for (int st = 0; st < STEPS; ++st) {
        const int i = wave * QUART + st * WAVE + lane;
        const bool valid = i < nvalid;
        const int sl = valid ? c[st] / W : 0;
        unsigned long long peers = __ballot(valid);
        for (int k = 0; k < nbits; ++k) {
            const bool one = (sl >> k) & 1;
            const unsigned long long m = __ballot(valid && one);
            peers &= one ? m : ~m;
        }
        int li = 0;
        if (valid) li = woff[wave][sl] + __popcll(peers & below);
        __builtin_amdgcn_wave_barrier();
        if (valid && (peers & below) == 0) woff[wave][sl] += __popcll(peers);
        __builtin_amdgcn_wave_barrier();
        if (valid) {
            s_val[li] = v[st];
            s_col[li] = (unsigned short)(c[st] - sl * W);
            s_row[li] = r[st];
            s_idx[li] = (unsigned short)i;
            s_slab[li] = (unsigned short)sl;
        }
    }
    __syncthreads();
    for (int i = tid; i < nvalid; i += 256) {
        const int sl = s_slab[i];
        const int dst = gbase[sl] + (i - lbase[sl]);
        svals[slab_value_index<SlabOf<T>::G>(dst)] = s_val[i];
        scol[dst] = s_col[i];
        srow[dst] = s_row[i];
        src[dst] = (int)(p0 + s_idx[i]);
    }
}

// Pairs.  One wave per chunk; slot j = chunk * CH + it * 64 + lane (it = 0 .. 7), so that the rows of the slots are read
// with full-width loads.  A slot starts a pair when it is the chunk's first or its row differs from the row of the slot
// before it (the lane below, or lane 63 of the round before); m[it] = the ballot of the starts of round it.
constexpr int SLAB_ROUNDS = SLAB_CH / WAVE;
__device__ __forceinline__ void chunk_starts(const int *__restrict__ srow, long long base, int lane,
                                             unsigned long long (&m)[SLAB_ROUNDS], int (&r)[SLAB_ROUNDS])
{
#pragma unroll
    for (int it = 0; it < SLAB_ROUNDS; ++it) r[it] = srow[base + it * WAVE + lane];
    int last = 0;
#pragma unroll
    for (int it = 0; it < SLAB_ROUNDS; ++it) {
        int prev = __shfl_up(r[it], 1, WAVE);
        if (lane == 0) prev = last;
        m[it] = __ballot((it == 0 && lane == 0) || r[it] != prev);
        last = rl(r[it], WAVE - 1);
    }
}

// cnt[c] = number of pairs of chunk c for c < nslots / CH (nslots = meta[0]), 0 for the entries up to `nmaxchunks`
// (the array is scanned over its whole length: its exclusive scan is chunk_pair).
__global__ __launch_bounds__(256) void k_slab_count(const int *__restrict__ meta, const int *__restrict__ srow,
                                                    int nmaxchunks, int *__restrict__ cnt)
{
    const int lane = threadIdx.x & (WAVE - 1);
    const int c = blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x / WAVE);
    if (c > nmaxchunks) return;
    const int nch = meta[0] / SLAB_CH;
    int total = 0;
    if (c < nch) {
        unsigned long long m[SLAB_ROUNDS];
        int r[SLAB_ROUNDS];
        chunk_starts(srow, (long long)c * SLAB_CH, lane, m, r);
#pragma unroll
        for (int it = 0; it < SLAB_ROUNDS; ++it) total += __popcll(m[it]);
    }
    if (lane == 0) cnt[c] = total;
}

// With chunk_pair = the exclusive scan of cnt: sets the end-of-pair bit of every pair's last slot (the slot before a
// start, and the chunk's last slot) and, for the first slot of every pair of a real row, leaves the pair's number + 1 at
// the CSR position the slot came from (pair_at, zero elsewhere), from which the row lists are formed.
// meta[1] = number of pairs.
__global__ __launch_bounds__(256) void k_slab_close(const int *__restrict__ meta_in, const int *__restrict__ srow,
                                                    const int *__restrict__ src, const int *__restrict__ chunk_pair,
                                                    unsigned short *__restrict__ scol, int *__restrict__ pair_at,
                                                    int *__restrict__ meta)
{
    const int lane = threadIdx.x & (WAVE - 1);
    const int c = blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x / WAVE);
    const int nch = meta_in[0] / SLAB_CH;
    if (c >= nch) return;
    const long long base = (long long)c * SLAB_CH;
    unsigned long long m[SLAB_ROUNDS];
    int r[SLAB_ROUNDS];
    chunk_starts(srow, base, lane, m, r);
    const int cp = chunk_pair[c];
    int before = 0;                                         // pairs of the chunk that start in earlier rounds
#pragma unroll
    for (int it = 0; it < SLAB_ROUNDS; ++it) {
        const long long j = base + it * WAVE + lane;
        const bool start = (m[it] >> lane) & 1ull;
        const bool end = lane < WAVE - 1 ? (m[it] >> (lane + 1)) & 1ull
                                         : (it < SLAB_ROUNDS - 1 ? m[it + 1 < SLAB_ROUNDS ? it + 1 : it] & 1ull : 1ull);
        if (end) scol[j] = (unsigned short)(scol[j] | 0x8000u);
        if (start && r[it] >= 0) {
            const int mine = cp + before + __popcll(m[it] & (~0ull >> (WAVE - 1 - lane))) - 1;     // this slot's pair
            pair_at[src[j]] = mine + 1;
        }
        before += __popcll(m[it]);
    }
    if (c == nch - 1 && lane == 0) meta[1] = chunk_pair[nch];
}

// R = exclusive scan of (pair_at != 0) over nnz + 1 entries: R[p] = number of pairs whose first slot comes from a CSR
// position below p.  Rows list their pairs in that order: qpos[r] = R[pos[r]], qidx[R[p]] = pair_at[p] - 1.
// meta[2] = number of listed pairs.
__global__ __launch_bounds__(256) void k_slab_rows(int rows, int nnz, const int *__restrict__ pos,
                                                   const int *__restrict__ R, const int *__restrict__ pair_at,
                                                   int *__restrict__ qpos, int *__restrict__ qidx,
                                                   int *__restrict__ meta)
{
    const long long g = (long long)blockIdx.x * 256 + threadIdx.x;
    if (g < nnz) {
        const int a = R[g];
        if (R[g + 1] != a) qidx[a] = pair_at[g] - 1;
    }
    if (g <= rows) qpos[g] = R[pos[g]];
    if (g == 0) meta[2] = R[nnz];
}

__global__ __launch_bounds__(256) void k_fill_int(int *__restrict__ p, long long n, int v)
{
    long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long stride = (long long)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = v;
}

hipError_t launch_fill_int(int32_t *p, int64_t n, int32_t v, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    PSK_LAUNCH(k_fill_int, dim3((unsigned)blocks), dim3(256), 0, s, p, (long long)n, v);
    return take_launch_status();
}

SlabBuildSpace carve_slab_build(void *base, int64_t rows, int64_t cols, int64_t nnz, int32_t W)
{
    (void)rows;
    SlabBuildSpace w;
    const int64_t S = (cols + W - 1) / W;
    const int64_t nblk = (nnz + BUILD_BT - 1) / BUILD_BT;
    const int64_t nmax = slab_max_slots(cols, nnz, W);
    char *p = static_cast<char *>(base);
    size_t o = 0;
    auto take = [&](size_t bytes) { char *q = p + o; o += align256(bytes); return q; };
    w.meta = reinterpret_cast<int32_t *>(take(256));
    w.tile_row = reinterpret_cast<int32_t *>(take((size_t)(nblk + 1) * 4));
    w.H = reinterpret_cast<int32_t *>(take((size_t)(S * nblk + 1) * 4));
    w.srow = reinterpret_cast<int32_t *>(take((size_t)(nmax + 1) * 4));
    w.src = reinterpret_cast<int32_t *>(take((size_t)(nmax + 1) * 4));
    w.F = reinterpret_cast<int32_t *>(take((size_t)(nmax / SLAB_CH + 2) * 4));       // pairs per chunk
    w.mark = reinterpret_cast<int32_t *>(take((size_t)(nnz + 1) * 4));
    w.pair_at = reinterpret_cast<int32_t *>(take((size_t)(nnz + 1) * 4));
    size_t tmp = scan_tmp_ints(S * nblk + 1);
    if (scan_tmp_ints(nnz + 1) > tmp) tmp = scan_tmp_ints(nnz + 1);
    w.scan_tmp = reinterpret_cast<int32_t *>(take(tmp * 4));
    w.bytes = o;
    return w;
}

// Enqueues the whole analysis on `s`.  When it has run, meta[0..2] = {slots, pairs, listed pairs}.
template <typename T>
static hipError_t launch_slab_build_t(int32_t rows, int32_t cols, int32_t nnz, const int32_t *pos, const int32_t *crd,
                                      const T *vals, const SlabBuildSpace &w, T *svals, uint16_t *scol,
                                      int32_t *chunk_pair, int32_t *slab_chunk, int32_t *qpos, int32_t *qidx,
                                      hipStream_t s)
{
    constexpr int W = SlabOf<T>::W;
    const int S = (int)(((int64_t)cols + W - 1) / W);
    const int nblk = (int)(((int64_t)nnz + BUILD_BT - 1) / BUILD_BT);
    const int64_t nmax = slab_max_slots(cols, nnz, W);
    unsigned short *scol_d = reinterpret_cast<unsigned short *>(scol);
    hipError_t e = launch_partition(rows, nnz, pos, BUILD_BT, 0, w.tile_row, s);
    if (e != hipSuccess) return e;
    const size_t lds = (size_t)S * 4;
    int nbits = 0;                                  // bits of a slab number
    while ((1 << nbits) < S) ++nbits;
    PSK_LAUNCH(k_slab_hist, dim3(nblk), dim3(256), (unsigned)lds, s, nnz, crd, W, S, nblk, w.H);
    PSK_LAUNCH(k_fill_int, dim3(1), dim3(64), 0, s, w.H + (long long)S * nblk, 1ll, 0);      // the scan's total slot
    launch_scan(w.H, w.H, (int64_t)S * nblk + 1, w.scan_tmp, false, s);
    PSK_LAUNCH(k_slab_bases, dim3(1), dim3(256), 0, s, w.H, S, nblk, slab_chunk, w.meta);
    PSK_LAUNCH(k_slab_pads<T>, dim3(S), dim3(64), 0, s, w.H, nblk, slab_chunk, svals, scol_d, w.srow, w.src);
    if (S <= STAGE_SLABS)
        PSK_LAUNCH(k_slab_scatter_staged<T>, dim3(nblk), dim3(256), 0, s, rows, nnz, pos, crd, vals, w.tile_row, w.H,
                   slab_chunk, S, nblk, nbits, svals, scol_d, w.srow, w.src);
    else
        PSK_LAUNCH(k_slab_scatter<T>, dim3(nblk), dim3(64), (unsigned)(lds + SCATTER_ROWS * 4), s, rows, nnz, pos, crd, vals,
                   w.tile_row, w.H, slab_chunk, S, nblk, nbits, svals, scol_d, w.srow, w.src);
    const int nmaxchunks = (int)(nmax / SLAB_CH);
    PSK_LAUNCH(k_slab_count, dim3((unsigned)(nmaxchunks / 4 + 1)), dim3(256), 0, s, w.meta, w.srow, nmaxchunks, w.F);
    launch_scan(w.F, chunk_pair, (int64_t)nmaxchunks + 1, w.scan_tmp, false, s);
    {
        int64_t blocks = ((int64_t)nnz + 1 + 255) / 256;
        if (blocks > 65536) blocks = 65536;
        PSK_LAUNCH(k_fill_int, dim3((unsigned)blocks), dim3(256), 0, s, w.pair_at, (long long)nnz + 1, 0);
    }
    PSK_LAUNCH(k_slab_close, dim3((unsigned)(nmaxchunks / 4 + 1)), dim3(256), 0, s, w.meta, w.srow, w.src, chunk_pair,
               scol_d, w.pair_at, w.meta);
    launch_scan(w.pair_at, w.mark, (int64_t)nnz + 1, w.scan_tmp, true, s);
    const int64_t span = ((int64_t)nnz > (int64_t)rows + 1 ? (int64_t)nnz : (int64_t)rows + 1);
    PSK_LAUNCH(k_slab_rows, dim3((unsigned)((span + 255) / 256)), dim3(256), 0, s, rows, nnz, pos, w.mark, w.pair_at,
               qpos, qidx, w.meta);
    return take_launch_status();
}

hipError_t launch_slab_build(int32_t rows, int32_t cols, int32_t nnz, const int32_t *pos, const int32_t *crd,
                             const float *vals, const SlabBuildSpace &w, float *svals, uint16_t *scol,
                             int32_t *chunk_pair, int32_t *slab_chunk, int32_t *qpos, int32_t *qidx, hipStream_t s)
{
    return launch_slab_build_t<float>(rows, cols, nnz, pos, crd, vals, w, svals, scol, chunk_pair, slab_chunk, qpos, qidx, s);
}

hipError_t launch_slab_build_f64(int32_t rows, int32_t cols, int32_t nnz, const int32_t *pos, const int32_t *crd,
                                 const double *vals, const SlabBuildSpace &w, double *svals, uint16_t *scol,
                                 int32_t *chunk_pair, int32_t *slab_chunk, int32_t *qpos, int32_t *qidx, hipStream_t s)
{
    return launch_slab_build_t<double>(rows, cols, nnz, pos, crd, vals, w, svals, scol, chunk_pair, slab_chunk, qpos, qidx, s);
}

#ifdef PSK_CU_TRACE
hipError_t cu_trace_set_slab(void *buf, unsigned records) { return cu_trace_set_here(buf, records); }
#endif

}  // namespace psk
