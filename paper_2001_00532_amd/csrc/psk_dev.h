// Device-side helpers shared by the kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace psk {

constexpr int WAVE = 64;
constexpr int NUM_XCD = 8;   // MI355X: 8 accelerator dies, workgroups are dealt to them round-robin

typedef int   v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));

// Streamed-once data (crd, vals): mark the loads non-temporal so they do not push
// the gathered operand out of L2.
template <typename T>
__device__ __forceinline__ T ld_stream(const T *p) { return __builtin_nontemporal_load(p); }

// DPP cross-lane move inside a row of 16 lanes; CTRL is the dpp_ctrl immediate.
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

// Sum over the 64 lanes of a wave; every lane receives the same bits.
// Butterfly: quad_perm xor1, quad_perm xor2, row_half_mirror, row_mirror (DPP),
// then xor16 / xor32 through the LDS crossbar.
__device__ __forceinline__ float wave_sum(float v)
{
    v += dpp_mov<0xB1>(v);    // quad_perm [1,0,3,2]
    v += dpp_mov<0x4E>(v);    // quad_perm [2,3,0,1]
    v += dpp_mov<0x141>(v);   // row_half_mirror
    v += dpp_mov<0x140>(v);   // row_mirror
    v += __shfl_xor(v, 16, WAVE);
    v += __shfl_xor(v, 32, WAVE);
    return v;
}

// Tile handled by a workgroup.  Workgroup b runs on die b % 8; give every die one
// contiguous eighth of the tiles so that the part of the dense operand a die
// gathers stays in that die's L2.  Returns -1 for the padding workgroups.
__device__ __forceinline__ int xcd_tile(int bid, int ntiles)
{
    const int per = (ntiles + NUM_XCD - 1) / NUM_XCD;
    const int t = (bid % NUM_XCD) * per + bid / NUM_XCD;
    return (bid / NUM_XCD < per && t < ntiles) ? t : -1;
}
__host__ __device__ __forceinline__ int xcd_grid(int ntiles) { return ((ntiles + NUM_XCD - 1) / NUM_XCD) * NUM_XCD; }

// LDS index skew: one group of `W` words of padding after every 32 words, so that
// per-lane runs whose starts are a multiple of 8/16/32 words apart spread over the banks.
template <int W>
__device__ __forceinline__ int skew(int i) { return i + (i >> 5) * W; }
template <int W>
constexpr int skewed_size(int n) { return n + ((n + 31) >> 5) * W; }

// ---- per-lane vectors of 1, 2 or 4 adjacent dense columns (SpMM, MTTKRP)
template <int VEC> struct VecT;
template <> struct VecT<1> { typedef float type; };
template <> struct VecT<2> { typedef v2f type; };
template <> struct VecT<4> { typedef v4f type; };

template <int VEC>
__device__ __forceinline__ void ld_vec(float (&d)[VEC], const float *p)
{
    typedef typename VecT<VEC>::type V;
    V v = *reinterpret_cast<const V *>(p);
    if constexpr (VEC == 1) d[0] = v;
    else {
#pragma unroll
        for (int i = 0; i < VEC; ++i) d[i] = v[i];
    }
}
template <int VEC>
__device__ __forceinline__ void st_vec(float *p, const float (&s)[VEC])
{
    typedef typename VecT<VEC>::type V;
    V v;
    if constexpr (VEC == 1) v = s[0];
    else {
#pragma unroll
        for (int i = 0; i < VEC; ++i) v[i] = s[i];
    }
    __builtin_nontemporal_store(v, reinterpret_cast<V *>(p));
}

// ---- per-workgroup trace (only in the instrumented build, -DPSK_CU_TRACE): every workgroup of a traced kernel
// records its start and end on the 100 MHz wall clock and the compute unit it ran on (HW_ID: cu, sh, se;
// XCC_ID: die) into a caller-supplied buffer of 3 x 64 bits per workgroup, from which the host forms each
// CU's busy time.  Each translation unit has its own copy of the pointer; psk_cu_trace_set sets them all.
#ifdef PSK_CU_TRACE
static __device__ unsigned long long *g_cu_trace = nullptr;
static __device__ unsigned g_cu_trace_records = 0;
struct WorkgroupTrace {
    unsigned long long t0;
    __device__ WorkgroupTrace() : t0(wall_clock64()) {}
    __device__ ~WorkgroupTrace()
    {
        if ((threadIdx.x & (WAVE - 1)) == 0 && g_cu_trace && blockIdx.x < g_cu_trace_records) {
            unsigned long long *r = g_cu_trace + 3ull * blockIdx.x;
            atomicMax(r + 1, (unsigned long long)wall_clock64());      // a workgroup ends with its last wave
            if (threadIdx.x == 0) {
                const unsigned hw = __builtin_amdgcn_s_getreg((15 << 11) | (0 << 6) | 4);     // HW_ID[15:0]
                const unsigned xcc = __builtin_amdgcn_s_getreg((3 << 11) | (0 << 6) | 20);    // XCC_ID[3:0]
                r[0] = t0;
                r[2] = (unsigned long long)hw | ((unsigned long long)xcc << 32);
            }
        }
    }
};
inline hipError_t cu_trace_set_here(void *buf, unsigned records)
{
    hipError_t e = hipMemcpyToSymbol(HIP_SYMBOL(g_cu_trace), &buf, sizeof(buf));
    if (e == hipSuccess) e = hipMemcpyToSymbol(HIP_SYMBOL(g_cu_trace_records), &records, sizeof(records));
    return e;
}
#define PSK_TRACE_WORKGROUP() WorkgroupTrace psk_trace_guard_
#else
#define PSK_TRACE_WORKGROUP() do { } while (0)
#endif

// Gathering x for four consecutive positions held by one lane.
//
// The vector-memory address unit takes about one clock per active lane for a gather whatever the
// width of the access (4, 8 or 16 bytes per lane cost the same), so the cheapest gather is the one
// with the fewest lane requests.  Positions whose columns are contiguous (c, c+1, ...: stencils,
// bands, dense blocks) can be served by one 16-byte load of their lane.  run_plan() looks at a lane's
// four columns: run A starts at position 0, run B right after it; if A and B together cover all four
// positions two wide loads replace four narrow ones.  The choice is made per wave (one ballot) so that
// both variants stay straight-line code with every load issued before the first use; unstructured
// matrices never take the wide path and keep their 4-byte gathers.
typedef float v4f_u __attribute__((ext_vector_type(4), aligned(4)));
struct RunPlan { int lenA; int colB; bool ok; };
__device__ __forceinline__ RunPlan run_plan(v4i c, int cols)
{
    const bool e1 = c.y == c.x + 1, e2 = c.z == c.y + 1, e3 = c.w == c.z + 1;
    RunPlan p;
    p.lenA = e1 ? (e2 ? (e3 ? 4 : 3) : 2) : 1;
    p.colB = p.lenA == 1 ? c.y : (p.lenA == 2 ? c.z : c.w);
    const bool covered = p.lenA >= 3 || (p.lenA == 2 && e3) || (p.lenA == 1 && e2 && e3);
    p.ok = covered && c.x <= cols - 4 && p.colB <= cols - 4;
    return p;
}
__device__ __forceinline__ void run_select(const RunPlan &p, v4f_u wA, v4f_u wB, float (&g)[4])
{
    g[0] = wA.x;
    g[1] = p.lenA >= 2 ? wA.y : wB.x;
    g[2] = p.lenA >= 3 ? wA.z : (p.lenA == 2 ? wB.x : wB.y);
    g[3] = p.lenA == 4 ? wA.w : (p.lenA == 3 ? wB.x : (p.lenA == 2 ? wB.y : wB.z));
}

__device__ __forceinline__ int   rl(int v, int lane)   { return __builtin_amdgcn_readlane(v, lane); }
__device__ __forceinline__ float rl(float v, int lane) { return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane)); }

}  // namespace psk
