// Shape-generic block-sparse attention over the selected key blocks (paper Eq. 2-3).
//
// One workgroup per (sequence, query head, query block); each wave owns query rows
// wave, wave+4, ... and walks the selected keys 64 at a time: one key per lane for the
// scores, an online softmax across the wave, then the probability-weighted value rows
// with the lanes spread over the channels.  fp32 arithmetic throughout.  The tuned kernels
// (attn_mfma.hip, attn_decode.hip) cover the benchmark shapes; this one covers the rest.
#include "common.h"
#include "launch.h"

namespace hipattn {

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void attn_generic_kernel(KParams p)
{
    constexpr int CPL = D / 64;  // output channels per lane
    extern __shared__ float q_s[];  // [bq][D]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t unit = blockIdx.x;
    const int qb = (int)(unit % p.nqb);
    const int h = (int)((unit / p.nqb) % p.hq);
    const int b = (int)(unit / ((int64_t)p.nqb * p.hq));
    const int hk = h / p.g;
    const int kb = p.kb, bk = p.bk;
    const int kv_len = p.kv_lens ? p.kv_lens[b] : p.max_kv_len;
    const int row0 = qb * p.bq;
    const int n_rows = min(p.bq, p.q_len - row0);
    const int pos0 = kv_len - p.q_len + row0;
    const int32_t *idx = p.idx_in + unit * kb;

    const T *Qb = (const T *)p.Q + (int64_t)b * p.qs_b + (int64_t)h * p.qs_h + (int64_t)row0 * p.qs_r;
    for (int i = tid; i < n_rows * D; i += kThreads) q_s[i] = ld_f32(Qb + (int64_t)(i / D) * p.qs_r + (i % D));
    __syncthreads();

    const T *Kbase = (const T *)p.K, *Vbase = (const T *)p.V, *Kback = (const T *)p.Kback, *Vback = (const T *)p.Vback;
    T *Ob = (T *)p.O + (int64_t)b * p.os_b + (int64_t)h * p.os_h + (int64_t)row0 * p.os_r;
    const int n_sel = kb * bk;

    for (int m = wave; m < n_rows; m += kThreads / 64) {
        const float *qrow = q_s + m * D;
        float m_run = -INFINITY, l_run = 0.f, acc[CPL];
#pragma unroll
        for (int c = 0; c < CPL; ++c) acc[c] = 0.f;

        // keys of this row: [0, vis) are admissible; the window takes [w0, vis), the sink takes
        // [0, ns) below the window, the selected blocks contribute what lies in [ns, w0)
        const int vis = min(pos0 + m + 1, kv_len);
        const int w0 = max(vis - p.n_window, 0);
        const int ns = min(p.n_sink, w0);
        const int n_keys = vis > 0 ? n_sel + ns + (vis - w0) : 0;

        for (int base = 0; base < n_keys; base += 64) {
            const int ki = base + lane;
            bool valid = ki < n_keys;
            int t = 0;
            if (valid) {
                if (ki < n_sel) {
                    const int j = ki / bk, n = ki - j * bk;
                    const int first = idx[j];
                    valid = first >= 0 && first < kv_len;
                    t = valid ? first + n : 0;
                    valid = valid && t >= ns && t < w0;
                } else if (ki < n_sel + ns) {
                    t = ki - n_sel;
                } else {
                    t = w0 + (ki - n_sel - ns);
                }
            }
            int64_t off = 0;
            bool miss = false;
            float s = -INFINITY;
            if (valid) {
                off = kv_row_offset(p, b, hk, t, miss);
                const T *krow = (miss ? Kback : Kbase) + off;
                float dot = 0.f;
                for (int c = 0; c < D; ++c) dot = fmaf(qrow[c], ld_f32(krow + c), dot);
                s = dot * p.sm_scale;
            }
            const float cmax = wave_max(s);
            if (cmax == -INFINITY) continue;  // no admissible key among these 64 (wave-uniform)
            const float m_new = fmaxf(m_run, cmax);
            const float alpha = expf(m_run - m_new);  // exp(-inf) = 0 on the first chunk
            const float pr = valid ? expf(s - m_new) : 0.f;
            l_run = l_run * alpha + wave_sum(pr);
#pragma unroll
            for (int c = 0; c < CPL; ++c) acc[c] *= alpha;
            const uint64_t live = __ballot(valid);
            for (int src = 0; src < 64; ++src) {
                if (!((live >> src) & 1)) continue;
                const float ps = __shfl(pr, src, 64);
                const int64_t so = __shfl((long long)off, src, 64);
                const T *vrow = (__shfl((int)miss, src, 64) ? Vback : Vbase) + so;
#pragma unroll
                for (int c = 0; c < CPL; ++c) acc[c] = fmaf(ps, ld_f32(vrow + lane + 64 * c), acc[c]);
            }
            m_run = m_new;
        }
        const float inv = l_run > 0.f ? 1.f / l_run : 0.f;
#pragma unroll
        for (int c = 0; c < CPL; ++c) st_f32(Ob + (int64_t)m * p.os_r + lane + 64 * c, acc[c] * inv);
    }
}

hipError_t launch_attn_generic(const KParams &p, bool bf16, hipStream_t st)
{
    const int64_t units = (int64_t)p.batch * p.hq * p.nqb;
    if (units == 0) return hipSuccess;
    const size_t smem = (size_t)p.bq * p.d * sizeof(float);
    dim3 grid((unsigned)units), block(kThreads);
    if (bf16) {
        if (p.d == 64) hipLaunchKernelGGL((attn_generic_kernel<bf16_t, 64>), grid, block, smem, st, p);
        else hipLaunchKernelGGL((attn_generic_kernel<bf16_t, 128>), grid, block, smem, st, p);
    } else {
        if (p.d == 64) hipLaunchKernelGGL((attn_generic_kernel<float, 64>), grid, block, smem, st, p);
        else hipLaunchKernelGGL((attn_generic_kernel<float, 128>), grid, block, smem, st, p);
    }
    return hipGetLastError();
}

}  // namespace hipattn
