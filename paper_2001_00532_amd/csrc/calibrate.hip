// Calibration kernels: not part of any product.  They measure, on the machine at hand, the three rates the
// design argues with -- a read-only stream, a gather of 4-byte words from a table in global memory, and the
// same gather from a table held in LDS -- so that the bounds quoted for the product kernels can be
// reproduced with `bench.py --workload stream_read | gather | gather_lds` and rocprofv3.
#include "../../include/psk.h"
#include "psk_dev.h"
#include "psk_internal.h"

namespace psk {

// Every thread reads 16 bytes per step with non-temporal loads, grid-stride; the sums keep the loads alive.
__global__ __launch_bounds__(256) void k_cal_stream_read(const v4f *__restrict__ src, long long n16, float *__restrict__ sink)
{
    float acc = 0.0f;
    const long long stride = (long long)gridDim.x * 256 * 4;
    long long i = (long long)blockIdx.x * 256 * 4 + threadIdx.x;
    for (; i + 3 * 256 < n16; i += stride) {
        const v4f a = ld_stream(src + i), b = ld_stream(src + i + 256), c = ld_stream(src + i + 512), d = ld_stream(src + i + 768);
        acc += a.x + b.y + c.z + d.w;
    }
    for (; i < n16; i += 256) acc += ld_stream(src + i).x;
    if (acc == 123456.789f) sink[0] = acc;       // practically never true: nothing is written
}

// 2048 gathers per workgroup, 8 per thread, indices streamed with 16-byte non-temporal loads (the access
// pattern of the CSR tile kernel without its values and row logic); one float per thread is written.
__global__ __launch_bounds__(256) void k_cal_gather(const int *__restrict__ idx, const float *__restrict__ table,
                                                    float *__restrict__ out, long long n)
{
    const long long base = (long long)blockIdx.x * 2048;
    if (base + 2048 > n) return;
    v4i c[2];
#pragma unroll
    for (int g = 0; g < 2; ++g) c[g] = ld_stream(reinterpret_cast<const v4i *>(idx + base + (g * 256 + threadIdx.x) * 4));
    float s = 0.0f;
#pragma unroll
    for (int g = 0; g < 2; ++g) { s += table[c[g].x]; s += table[c[g].y]; s += table[c[g].z]; s += table[c[g].w]; }
    out[(long long)blockIdx.x * 256 + threadIdx.x] = s;
}

// The same number of gathers from a table of at most kSlabCols floats that each workgroup first copies into
// LDS; indices are 16-bit, 8 per lane and step (one 16-byte load), as in the column-slab pair kernel.
__global__ __launch_bounds__(1024) void k_cal_gather_lds(const unsigned short *__restrict__ idx, const float *__restrict__ table,
                                                         int table_n, float *__restrict__ out, long long n, int steps)
{
    __shared__ float xs[kSlabCols];
    for (int i = threadIdx.x; i < table_n; i += 1024) xs[i] = table[i];
    __syncthreads();
    float s = 0.0f;
    const long long base = (long long)blockIdx.x * steps * 8192;
    for (int t = 0; t < steps; ++t) {
        const long long b = base + (long long)t * 8192 + threadIdx.x * 8;
        if (b + 8 > n) break;
        const v4i q = ld_stream(reinterpret_cast<const v4i *>(idx + b));
        const unsigned w[4] = {(unsigned)q.x, (unsigned)q.y, (unsigned)q.z, (unsigned)q.w};
#pragma unroll
        for (int j = 0; j < 8; ++j) s += xs[(j & 1) ? (w[j >> 1] >> 16) : (w[j >> 1] & 0xffffu)];
    }
    out[(long long)blockIdx.x * 1024 + threadIdx.x] = s;
}

}  // namespace psk

using namespace psk;

extern "C" {

int psk_calibrate_stream_read(const void *src, size_t bytes, float *sink, void *stream)
{
    if (!src || !sink) return PSK_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(src) & 15) || bytes < 16) return PSK_ERR_ALIGNMENT;
    const long long n16 = (long long)(bytes / 16);
    long long blocks = (n16 + 1023) / 1024;
    if (blocks > 256 * 32) blocks = 256 * 32;
    PSK_LAUNCH(k_cal_stream_read, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
               static_cast<const v4f *>(src), n16, sink);
    return take_launch_status() == hipSuccess ? PSK_OK : PSK_ERR_HIP;
}

int psk_calibrate_gather(const float *table, int64_t table_elems, const int32_t *idx, int64_t n, float *out, void *stream)
{
    if (!table || !idx || !out) return PSK_ERR_NULL;
    if (table_elems <= 0 || n < 2048 || n % 2048) return PSK_ERR_SIZE;
    if (reinterpret_cast<uintptr_t>(idx) & 15) return PSK_ERR_ALIGNMENT;
    PSK_LAUNCH(k_cal_gather, dim3((unsigned)(n / 2048)), dim3(256), 0, static_cast<hipStream_t>(stream), idx, table, out,
               (long long)n);
    return take_launch_status() == hipSuccess ? PSK_OK : PSK_ERR_HIP;
}

int psk_calibrate_gather_lds(const float *table, int32_t table_elems, const uint16_t *idx, int64_t n, float *out,
                             void *stream)
{
    if (!table || !idx || !out) return PSK_ERR_NULL;
    if (table_elems <= 0 || table_elems > kSlabCols || n < 8192 || n % 8192) return PSK_ERR_SIZE;
    if (reinterpret_cast<uintptr_t>(idx) & 15) return PSK_ERR_ALIGNMENT;
    const long long chunks = n / 8192;
    const int grid = chunks < 256 ? (int)chunks : 256;
    const int steps = (int)((chunks + grid - 1) / grid);
    PSK_LAUNCH(k_cal_gather_lds, dim3(grid), dim3(1024), 0, static_cast<hipStream_t>(stream),
               reinterpret_cast<const unsigned short *>(idx), table, table_elems, out, (long long)n, steps);
    return take_launch_status() == hipSuccess ? PSK_OK : PSK_ERR_HIP;
}

}  // extern "C"
