// Test and measurement aids (libhipattn_aux.so), not part of the method and not part of the product
// library: an LDS poisoner for the GPU tests, and probes of what this GPU sustains (device copy, read
// sweep, back-to-back bf16 MFMA, gather of key-block-sized runs from a working set of a given size), so
// that roofline fractions can be quoted against measured ceilings next to the published ones.
#include "../../include/hipattn_aux.h"

#include <hip/hip_runtime.h>

namespace {

constexpr int kThreads = 256;

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
int launch_result(hipError_t e) { return e == hipSuccess ? 0 : -1000 - (int)e; }

__global__ __launch_bounds__(kThreads) void poison_lds_kernel(uint32_t pattern)
{
    extern __shared__ uint32_t lds_words[];
    volatile uint32_t *w = lds_words;  // volatile: the stores are the whole point
    for (int i = threadIdx.x; i < 65536 / 4; i += kThreads) w[i] = pattern;
}

// 16 bytes per lane and step, grid-stride over n16 16-byte units
__global__ __launch_bounds__(kThreads) void probe_copy_kernel(u32x4_t *__restrict__ dst, const u32x4_t *__restrict__ src,
                                                              int64_t n16)
{
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n16; i += stride)
        dst[i] = __builtin_nontemporal_load(src + i);
}

// read-only sweep: every lane folds its 16-byte units into one word and writes it at the end
__global__ __launch_bounds__(kThreads) void probe_read_kernel(uint32_t *__restrict__ out, const u32x4_t *__restrict__ src,
                                                              int64_t n16)
{
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    u32x4_t acc = {0u, 0u, 0u, 0u};
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n16; i += stride)
        acc ^= __builtin_nontemporal_load(src + i);
    out[(int64_t)blockIdx.x * kThreads + threadIdx.x] = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
}

// every wave issues iters * 4 independent 32x32x16 bf16 MFMAs on register operands
__global__ __launch_bounds__(kThreads) void probe_mfma_kernel(float *__restrict__ out, int iters)
{
    bf16x8_t a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(float)((threadIdx.x + i) & 3);
        b[i] = (__bf16)(float)((threadIdx.x * 3 + i) & 1);
    }
    f32x16_t c0 = {}, c1 = {}, c2 = {}, c3 = {};
    for (int it = 0; it < iters; ++it) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
    out[(int64_t)blockIdx.x * kThreads + threadIdx.x] = s;
}

__device__ __forceinline__ uint32_t mix32(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}

// The access pattern of the two attention kernels without their arithmetic: every wave reads `tiles`
// tiles of 32 rows of 256 bytes; a tile is 32 / run runs of `run` consecutive rows whose first row is
// drawn (hashed from workgroup, wave, tile and run number) among the rows of this workgroup's slice of
// the buffer.  16 lanes read one row (16 bytes each), so one wave-wide load covers 4 rows and 8 loads a
// tile; 4 tiles are in flight.  Workgroup w works on slice w % slices (slices = 8 pins a slice to an XCD
// and its L2, as the kernels pin a kv head).
__global__ __launch_bounds__(kThreads) void probe_gather_kernel(uint32_t *__restrict__ out, const char *__restrict__ src,
                                                                uint32_t rows_per_slice, int slices, int log_run, int tiles)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lg = lane >> 4, lc = lane & 15;
    const char *base = src + (int64_t)(blockIdx.x % slices) * rows_per_slice * 256;
    const uint32_t run = 1u << log_run, n_runs = rows_per_slice >> log_run;
    const uint32_t salt = mix32((blockIdx.x * 4u + wave) * 0x9e3779b9u + 1u);
    u32x4_t acc = {0u, 0u, 0u, 0u};
    for (int t = 0; t < tiles; t += 4) {
        u32x4_t v[4][8];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t row_in_tile = 4u * j + lg;                 // 0..31
                const uint32_t r = mix32(salt + ((uint32_t)(t + u) << 6) + (row_in_tile >> log_run));
                const uint32_t first = (uint32_t)(((uint64_t)r * n_runs) >> 32) << log_run;
                const uint32_t row = first + (row_in_tile & (run - 1));
                v[u][j] = *(const u32x4_t *)(base + (int64_t)row * 256 + lc * 16);
            }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc ^= v[u][j];
    }
    out[(int64_t)blockIdx.x * kThreads + threadIdx.x] = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
}

}  // namespace

extern "C" {

int hip_attn_poison_lds(uint32_t pattern, void *stream)
{
    // 2 workgroups of 64 KB fit a compute unit: 8192 workgroups sweep all 256 units many times
    hipLaunchKernelGGL(poison_lds_kernel, dim3(8192), dim3(kThreads), 65536, static_cast<hipStream_t>(stream), pattern);
    return launch_result(hipGetLastError());
}

int hip_attn_probe_copy(void *dst, const void *src, size_t bytes, void *stream)
{
    if (!dst || !src) return -1;
    if (!aligned16(dst) || !aligned16(src) || bytes % 16) return -7;
    const int64_t n16 = (int64_t)(bytes / 16);
    if (n16 == 0) return 0;
    const int64_t want = (n16 + kThreads - 1) / kThreads;
    const unsigned grid = (unsigned)(want < 256 * 32 ? want : 256 * 32);
    hipLaunchKernelGGL(probe_copy_kernel, dim3(grid), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                       (u32x4_t *)dst, (const u32x4_t *)src, n16);
    return launch_result(hipGetLastError());
}

int hip_attn_probe_read(uint32_t *out, const void *src, size_t bytes, void *stream)
{
    if (!out || !src) return -1;
    if (!aligned16(src) || bytes % 16) return -7;
    hipLaunchKernelGGL(probe_read_kernel, dim3(HIP_ATTN_PROBE_READ_WORDS / kThreads), dim3(kThreads), 0,
                       static_cast<hipStream_t>(stream), out, (const u32x4_t *)src, (int64_t)(bytes / 16));
    return launch_result(hipGetLastError());
}

int hip_attn_probe_mfma(float *out, int32_t workgroups, int32_t iters, void *stream)
{
    if (!out) return -1;
    if (workgroups <= 0 || iters <= 0) return -2;
    hipLaunchKernelGGL(probe_mfma_kernel, dim3((unsigned)workgroups), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                       out, iters);
    return launch_result(hipGetLastError());
}

int hip_attn_probe_gather(uint32_t *out, const void *src, size_t bytes, int32_t slices, int32_t run_rows,
                          int32_t workgroups, int32_t tiles, void *stream)
{
    if (!out || !src) return -1;
    if (!aligned16(src)) return -7;
    if (slices <= 0 || workgroups <= 0 || tiles <= 0 || tiles % 4) return -2;
    int log_run = 0;
    while ((1 << log_run) < run_rows) ++log_run;
    if (run_rows <= 0 || (1 << log_run) != run_rows || run_rows > 32) return -2;
    const size_t rows = bytes / 256 / (size_t)slices;
    if (rows < 32 || rows > 0xffffffffu) return -2;
    hipLaunchKernelGGL(probe_gather_kernel, dim3((unsigned)workgroups), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                       out, (const char *)src, (uint32_t)rows, slices, log_run, tiles);
    return launch_result(hipGetLastError());
}

}  // extern "C"
