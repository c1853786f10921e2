// Top-r approximation of the mask-estimation scores (paper appendix "Top-r Approximation"): a query
// row's products run over the r channels in which its |q| is largest.  This pre-pass writes a copy of Q
// with every other channel zeroed into the caller's workspace (dense [batch, n_q_heads, q_len, head_dim]);
// the mask-estimation kernels then read that copy and need no change.
//
// One wave per row, lane l holds channels l, l + 64 (head_dim 128).  The r-th largest magnitude is found
// bit by bit on the magnitudes' bit patterns (they order like the values); channels above it stay, equal
// ones stay in channel order while room is left.
#include "common.h"
#include "launch.h"

namespace hipattn {

template <typename T> struct mag_bits;
template <> struct mag_bits<float> {
    static constexpr int top_bit = 30;
    static __device__ __forceinline__ uint32_t of(float v) { return __float_as_uint(v) & 0x7fffffffu; }
};
template <> struct mag_bits<bf16_t> {
    static constexpr int top_bit = 14;
    static __device__ __forceinline__ uint32_t of(bf16_t v) { return v & 0x7fffu; }
};

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void topr_mask_kernel(KParams p, T *__restrict__ dst, int64_t n_rows)
{
    constexpr int CPL = D / 64;
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (row >= n_rows) return;
    const int i = (int)(row % p.q_len);
    const int h = (int)((row / p.q_len) % p.hq);
    const int b = (int)(row / ((int64_t)p.q_len * p.hq));
    const T *src = (const T *)p.Q + (int64_t)b * p.qs_b + (int64_t)h * p.qs_h + (int64_t)i * p.qs_r;
    T v[CPL];
    uint32_t a[CPL];
#pragma unroll
    for (int j = 0; j < CPL; ++j) {
        v[j] = src[lane + 64 * j];
        a[j] = mag_bits<T>::of(v[j]);
    }
    uint32_t thr = 0;
    for (int bit = mag_bits<T>::top_bit; bit >= 0; --bit) {
        const uint32_t cand = thr | (1u << bit);
        int cnt = 0;
#pragma unroll
        for (int j = 0; j < CPL; ++j) cnt += __popcll(__ballot(a[j] >= cand));
        if (cnt >= p.top_r) thr = cand;
    }
    int above = 0;
#pragma unroll
    for (int j = 0; j < CPL; ++j) above += __popcll(__ballot(a[j] > thr));
    int ties_before = 0;
#pragma unroll
    for (int j = 0; j < CPL; ++j) {
        const uint64_t tie = __ballot(a[j] == thr);
        const int mine = ties_before + __popcll(tie & ((1ull << lane) - 1));
        const bool keep = a[j] > thr || (a[j] == thr && above + mine < p.top_r);
        dst[row * D + lane + 64 * j] = keep ? v[j] : T(0);
        ties_before += __popcll(tie);
    }
}

hipError_t launch_topr_mask(const KParams &p, bool bf16, void *dst, hipStream_t st)
{
    const int64_t n_rows = (int64_t)p.batch * p.hq * p.q_len;
    if (n_rows == 0) return hipSuccess;
    const int64_t blocks = (n_rows + kThreads / 64 - 1) / (kThreads / 64);
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    dim3 grid((unsigned)blocks), block(kThreads);
    if (bf16) {
        if (p.d == 64) hipLaunchKernelGGL((topr_mask_kernel<bf16_t, 64>), grid, block, 0, st, p, (bf16_t *)dst, n_rows);
        else hipLaunchKernelGGL((topr_mask_kernel<bf16_t, 128>), grid, block, 0, st, p, (bf16_t *)dst, n_rows);
    } else {
        if (p.d == 64) hipLaunchKernelGGL((topr_mask_kernel<float, 64>), grid, block, 0, st, p, (float *)dst, n_rows);
        else hipLaunchKernelGGL((topr_mask_kernel<float, 128>), grid, block, 0, st, p, (float *)dst, n_rows);
    }
    return hipGetLastError();
}

}  // namespace hipattn
