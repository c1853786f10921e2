// Pages read by the sparse attention of a call (token bank of paper Sec. 3.3): a byte map for the cache
// manager.  The set follows from the index array and the sink / window sizes alone, so it is written by
// this small kernel after the attention kernel instead of from inside its gather loop.
#include "common.h"
#include "launch.h"

namespace hipattn {

// One wave per (sequence, query head, query block).
__global__ __launch_bounds__(kThreads) void touch_attn_kernel(KParams p, int64_t units)
{
    const int lane = threadIdx.x & 63;
    const int64_t unit = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (unit >= units) return;
    const int qb = (int)(unit % p.nqb);
    const int b = (int)(unit / ((int64_t)p.nqb * p.hq));
    const int kv_len = p.kv_lens ? p.kv_lens[b] : p.max_kv_len;
    const int row0 = qb * p.bq;
    const int n_rows = min(p.bq, p.q_len - row0);
    const int pos0 = kv_len - p.q_len + row0, pos_last = pos0 + n_rows - 1;
    if (pos_last < 0 || kv_len <= 0) return;  // no row of this block exists yet
    // keys [0, vis_last) are visible to the block's last row, [0, vis_first) to its first existing row
    const int vis_last = min(pos_last + 1, kv_len), vis_first = min(max(pos0, 0) + 1, kv_len);
    const int32_t *idx = p.idx_in + unit * p.kb;
    // selected blocks: read if at least their first key is visible to the last row
    for (int j = lane; j < p.kb; j += 64) {
        const int first = idx[j];
        if (first >= 0 && first < vis_last) {
            touch_page(p, b, first);
            touch_page(p, b, min(first + p.bk, vis_last) - 1);
        }
    }
    // sink keys [0, ns) and the union of the rows' windows [w0, vis_last)
    const int ns = min(p.n_sink, vis_last);
    for (int pg = lane; ns > 0 && pg <= logical_page(p, ns - 1); pg += 64) p.touched[(int64_t)b * p.max_pages + pg] = 1;
    if (p.n_window > 0) {
        const int w0 = max(vis_first - p.n_window, 0);
        for (int pg = logical_page(p, w0) + lane; pg <= logical_page(p, vis_last - 1); pg += 64)
            p.touched[(int64_t)b * p.max_pages + pg] = 1;
    }
}

hipError_t launch_touch_attn(const KParams &p, hipStream_t st)
{
    const int64_t units = (int64_t)p.batch * p.hq * p.nqb;
    if (units == 0 || !p.touched) return hipSuccess;
    const int64_t blocks = (units + kThreads / 64 - 1) / (kThreads / 64);
    hipLaunchKernelGGL(touch_attn_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, st, p, units);
    return hipGetLastError();
}

}  // namespace hipattn
