// Measurement aids, not part of the method: what this GPU sustains on a plain device copy and on
// back-to-back bf16 MFMA instructions, so that roofline fractions can be quoted against measured
// ceilings next to the published ones.
#include "common.h"
#include "launch.h"

namespace hipattn {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

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

hipError_t launch_probe_copy(void *dst, const void *src, int64_t bytes, hipStream_t st)
{
    const int64_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    const int64_t want = (n16 + kThreads - 1) / kThreads;
    const unsigned grid = (unsigned)(want < 256 * 32 ? want : 256 * 32);
    hipLaunchKernelGGL(probe_copy_kernel, dim3(grid), dim3(kThreads), 0, st, (u32x4_t *)dst, (const u32x4_t *)src, n16);
    return hipGetLastError();
}

hipError_t launch_probe_read(uint32_t *out, const void *src, int64_t bytes, hipStream_t st)
{
    hipLaunchKernelGGL(probe_read_kernel, dim3(kProbeReadGrid), dim3(kThreads), 0, st, out, (const u32x4_t *)src, bytes / 16);
    return hipGetLastError();
}

hipError_t launch_probe_mfma(float *out, int workgroups, int iters, hipStream_t st)
{
    hipLaunchKernelGGL(probe_mfma_kernel, dim3((unsigned)workgroups), dim3(kThreads), 0, st, out, iters);
    return hipGetLastError();
}

}  // namespace hipattn
