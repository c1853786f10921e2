// Block-sparse attention for single-query decode in bf16 (paper Eq. 2-3 for one query row
// per sequence; the sparse-attention step of Alg. 2).
//
// One wave per (sequence, query head).  A key row is read by D/8 lanes (16 bytes each),
// so a wave-wide load covers 64/(D/8) rows; each such lane group walks its own subset of the
// selected blocks with its own online-softmax state (running max, sum and 8 output channels
// per lane), loading the value row of a key right next to its key row.  The groups'
// states are merged at the end with a few cross-lane exchanges.  Everything is fp32 after
// the loads; HBM bound (K and V rows are touched exactly once).
#include "common.h"
#include "launch.h"

namespace hipattn {

// SPLIT = false: one wave per (sequence, head).  SPLIT = true (up to 8192 problems): one workgroup per
// (sequence, head), stage i of the block list goes to wave i % 4, the four partial softmax states
// are merged through LDS.
template <int BK, int D, int ROWS, bool PAGED, bool SPLIT>
__global__ __launch_bounds__(kThreads) void attn_decode_kernel(KParams p, int sub_shift)
{
    constexpr int LPR = D / 8, RPW = 64 / LPR;
    constexpr int U = ROWS / BK;  // blocks per lane group and stage: ROWS key + ROWS value row loads per lane, two stages in flight
    typedef uint32_t stage_t __attribute__((ext_vector_type(4 * U * BK)));
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // (uniform: what follows from it stays in scalar registers)
    const int grp = lane / LPR, lc = lane % LPR;
    const int64_t wg = SPLIT ? (int64_t)blockIdx.x : (int64_t)blockIdx.x * 4 + wave;
    if (wg >= (int64_t)p.batch * p.hq) return;
    const int b = (int)(wg / p.hq), h = (int)(wg % p.hq), hk = h / p.g;
    const int kb = p.kb;
    const int kv_len = p.kv_lens ? p.kv_lens[b] : p.max_kv_len;
    const int32_t *idx = p.idx_in + wg * kb;

    const uint4 qv = *(const uint4 *)((const bf16_t *)p.Q + (int64_t)b * p.qs_b + (int64_t)h * p.qs_h + lc * 8);
    const bf16_t *Kbase = (const bf16_t *)p.K, *Vbase = (const bf16_t *)p.V;
    const float c = p.sm_scale * 1.44269504088896340736f;

    float m_run = -INFINITY, l_run = 0.f, acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;

    // one stage = U blocks per lane group: BK key rows and BK value rows each, loaded
    // unconditionally (a block that does not count re-reads row 0 and gets probability 0).
    // Block list: the kb selected blocks, then the sink range, then the window range cut into
    // BK-aligned blocks.  Rows of a block count iff lo <= position < hi:
    //   selected [n_sink, w0), sink [0, ns), window [w0, kv_len), with w0 = kv_len - n_window.
    const int w0 = max(kv_len - p.n_window, 0);
    const int ns = min(p.n_sink, w0);
    const int nb_sink = (ns + BK - 1) / BK;
    const int win_first = (w0 / BK) * BK;
    const int nb_win = p.n_window > 0 ? (kv_len - win_first + BK - 1) / BK : 0;
    // key blocks of 8 or 16 rows are walked as 2 or 4 pieces of BK = 4 rows: kbv pieces in all
    const int kbv = kb << sub_shift;
    const int n_blocks = kbv + nb_sink + nb_win;

    // one stage = U blocks per lane group: BK key rows and BK value rows each, loaded
    // unconditionally (a block that does not count re-reads row 0 and gets probability 0).
    // okm[u]: bit n set iff row n of block u counts
    auto fetch = [&](int base, stage_t &kr, stage_t &vr, int (&okm)[U]) __attribute__((always_inline)) {
        int pg[U], first[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = base + u * RPW + grp;
            int f = -1, lo = 0, hi = 0;
            if (j < kbv) {
                f = idx[j >> sub_shift];
                if (f >= 0) f += (j & ((1 << sub_shift) - 1)) * BK;
                if (f >= kv_len) f = -1;
                lo = p.n_sink; hi = w0;
            } else if (j < kbv + nb_sink) {
                f = (j - kbv) * BK;
                hi = ns;
            } else if (j < n_blocks) {
                f = win_first + (j - kbv - nb_sink) * BK;
                lo = w0; hi = kv_len;
            }
            first[u] = f;
            int m = 0;
#pragma unroll
            for (int n = 0; n < BK; ++n) m |= (f >= 0 && f + n >= lo && f + n < hi) ? (1 << n) : 0;
            okm[u] = m;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) pg[u] = page_of_row<PAGED>(p, b, first[u] >= 0 ? first[u] : 0);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int f = first[u];
            const int64_t off = row_offset_in<PAGED>(p, b, hk, f >= 0 ? f : 0, page_in_pool(pg[u])) + lc * 8;
            // (a negative page-table entry names a page of the backing pools)
            const bf16_t *Kp = (const bf16_t *)pool_of(pg[u], Kbase, p.Kback), *Vp = (const bf16_t *)pool_of(pg[u], Vbase, p.Vback);
#pragma unroll
            for (int n = 0; n < BK; ++n) {
                const int dn = f >= 0 ? min(n, kv_len - 1 - f) : 0;
                const uint4 x = *(const uint4 *)(Kp + off + (int64_t)dn * p.ks_r);
                const uint4 y = *(const uint4 *)(Vp + off + (int64_t)dn * p.ks_r);
                const int q4 = 4 * (u * BK + n);
                kr[q4] = x.x; kr[q4 + 1] = x.y; kr[q4 + 2] = x.z; kr[q4 + 3] = x.w;
                vr[q4] = y.x; vr[q4 + 1] = y.y; vr[q4 + 2] = y.z; vr[q4 + 3] = y.w;
            }
        }
    };
    auto consume = [&](const stage_t &kr, const stage_t &vr, const int (&okm)[U]) __attribute__((always_inline)) {
        float s[U][BK], mx = -INFINITY;
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int n = 0; n < BK; ++n) {
                const int q4 = 4 * (u * BK + n);
                const float d = row_group_sum<LPR>(dot8_bf16(qv, make_uint4(kr[q4], kr[q4 + 1], kr[q4 + 2], kr[q4 + 3]))) * c;
                // the query is the last position of its sequence: no key is in its future
                s[u][n] = ((okm[u] >> n) & 1) ? d : -INFINITY;
                mx = fmaxf(mx, s[u][n]);
            }
        const float m_new = fmaxf(m_run, mx);
        const float m_safe = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);
        l_run *= alpha;
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] *= alpha;
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int n = 0; n < BK; ++n) {
                const float pr = __builtin_amdgcn_exp2f(s[u][n] - m_safe);
                l_run += pr;
                const int q4 = 4 * (u * BK + n);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    acc[2 * i] = fmaf(pr, __uint_as_float(vr[q4 + i] << 16), acc[2 * i]);
                    acc[2 * i + 1] = fmaf(pr, __uint_as_float(vr[q4 + i] & 0xffff0000u), acc[2 * i + 1]);
                }
            }
        m_run = m_new;
    };

    constexpr int STEP = RPW * U;                      // blocks per stage
    constexpr int STRIDE = (SPLIT ? 4 : 1) * STEP;     // distance between two stages of the same wave
    stage_t ka, va, kb2, vb2;
    int fa[U], fb[U];
    const int first_base = SPLIT ? wave * STEP : 0;
    if (first_base < n_blocks) fetch(first_base, ka, va, fa);
    for (int base = first_base; base < n_blocks; base += 2 * STRIDE) {
        const bool has_b = base + STRIDE < n_blocks;
        if (has_b) fetch(base + STRIDE, kb2, vb2, fb);
        consume(ka, va, fa);
        if (has_b) {
            if (base + 2 * STRIDE < n_blocks) fetch(base + 2 * STRIDE, ka, va, fa);
            consume(kb2, vb2, fb);
        }
    }

    // merge the lane groups' partial softmax states (same channels, different keys)
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) {
        const float m_o = __shfl_xor(m_run, off, 64), l_o = __shfl_xor(l_run, off, 64);
        const float m_new = fmaxf(m_run, m_o);
        const float m_safe = m_new == -INFINITY ? 0.f : m_new;
        const float a = __builtin_amdgcn_exp2f(m_run - m_safe), ao = __builtin_amdgcn_exp2f(m_o - m_safe);
        l_run = l_run * a + l_o * ao;
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = acc[i] * a + __shfl_xor(acc[i], off, 64) * ao;
        m_run = m_new;
    }
    if (SPLIT) {
        // lanes of group 0 of every wave hold that wave's state for channels lc*8 .. +8
        __shared__ float part_s[4][LPR][10];
        if (grp == 0) {
            part_s[wave][lc][0] = m_run;
            part_s[wave][lc][1] = l_run;
#pragma unroll
            for (int i = 0; i < 8; ++i) part_s[wave][lc][2 + i] = acc[i];
        }
        __syncthreads();
        if (wave != 0) return;
        if (grp == 0) {
#pragma unroll
            for (int w = 1; w < 4; ++w) {
                const float m_o = part_s[w][lc][0], l_o = part_s[w][lc][1];
                const float m_new = fmaxf(m_run, m_o);
                const float m_safe = m_new == -INFINITY ? 0.f : m_new;
                const float a = __builtin_amdgcn_exp2f(m_run - m_safe), ao = __builtin_amdgcn_exp2f(m_o - m_safe);
                l_run = l_run * a + l_o * ao;
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[i] = acc[i] * a + part_s[w][lc][2 + i] * ao;
                m_run = m_new;
            }
        }
    }
    if (grp == 0) {
        const float inv = l_run > 0.f ? 1.f / l_run : 0.f;
        uint4 o;
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            w[i] = (uint32_t)f32_to_bf16(acc[2 * i] * inv) | ((uint32_t)f32_to_bf16(acc[2 * i + 1] * inv) << 16);
        o = make_uint4(w[0], w[1], w[2], w[3]);
        *(uint4 *)((bf16_t *)p.O + (int64_t)b * p.os_b + (int64_t)h * p.os_h + lc * 8) = o;
    }
}

bool attn_decode_supported(const KParams &p, bool bf16)
{
    return bf16 && p.q_len == 1 && p.bq == 1 && (p.bk == 1 || p.bk == 2 || p.bk == 4 || p.bk == 8 || p.bk == 16);
}

hipError_t launch_attn_decode(const KParams &p, hipStream_t st)
{
    const int64_t waves = (int64_t)p.batch * p.hq;
    if (waves == 0) return hipSuccess;
    // up to 8192 problems: a workgroup per problem (four waves share its blocks); beyond that a wave per problem
    // (measured at 32 query heads, 512 keys: 3072 problems -11 %, 8192 -1 %, 16384 +3 %, 32768 +22 %)
    const bool split = waves <= 8192;
    dim3 grid((unsigned)(split ? waves : (waves + 3) / 4)), block(kThreads);
    const bool paged = p.page_table != nullptr;
    const int sub_shift = p.bk == 8 ? 1 : p.bk == 16 ? 2 : 0;  // blocks of 8 / 16 rows as pieces of 4
#define HIPATTN_LAUNCH(BKV, DV)                                                                        \
    do {                                                                                               \
        if (split && paged) hipLaunchKernelGGL((attn_decode_kernel<BKV, DV, 4, true, true>), grid, block, 0, st, p, sub_shift);         \
        else if (split) hipLaunchKernelGGL((attn_decode_kernel<BKV, DV, 4, false, true>), grid, block, 0, st, p, sub_shift);            \
        else if (paged) hipLaunchKernelGGL((attn_decode_kernel<BKV, DV, 4, true, false>), grid, block, 0, st, p, sub_shift);            \
        else hipLaunchKernelGGL((attn_decode_kernel<BKV, DV, 4, false, false>), grid, block, 0, st, p, sub_shift);                      \
    } while (0)
    if (p.d == 64) {
        if (p.bk == 1) HIPATTN_LAUNCH(1, 64);
        else if (p.bk == 2) HIPATTN_LAUNCH(2, 64);
        else HIPATTN_LAUNCH(4, 64);
    } else {
        if (p.bk == 1) HIPATTN_LAUNCH(1, 128);
        else if (p.bk == 2) HIPATTN_LAUNCH(2, 128);
        else HIPATTN_LAUNCH(4, 128);
    }
#undef HIPATTN_LAUNCH
    return hipGetLastError();
}

}  // namespace hipattn
