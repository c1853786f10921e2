// Hierarchical mask estimation for single-query decode in bf16 (paper Alg. 2: one run of
// Alg. 1 per step over the current context, with bq = 1).
//
// With one query row the branch scoring is vector x gathered-rows work: bandwidth bound, no
// use for the matrix cores.  Two forms (template parameter SPLIT, chosen by the number of problems): one
// WORKGROUP per (sequence, query head), or one WAVE per problem with the four waves of a workgroup being the
// query heads of one KV group when Hq/Hkv = 4.  Either way the heads of a KV group run next to each other, so in
// the first round, where they score the same representative blocks, their loads meet in the L1/L2 instead of
// going to HBM four times.
//   * a key row is read by D/8 lanes, 16 bytes each (a full 128-bit coalesced row segment),
//     multiplied with v_dot2_f32_bf16 and summed over the lanes with DPP adds;
//   * two stages of 8 row loads per lane alternate, so up to 16 KB per wave are in flight;
//   * scores -> LDS keys -> ordered threshold selection -> the problem's node list (wave per problem: private to
//     the wave, nothing redundant, no workgroup barrier anywhere);
//   * with the first or the last block as representative, one child of every node has the
//     node's own representative (left child / first block, right child / last block): its score is
//     the score that selected the node, carried over as a key, and from the second round on only the
//     other child is gathered and scored - about half the memory traffic.  With the centre representative
//     the same holds in the final round (every node one or two blocks long: a one-block node is its own
//     representative, the right half of a two-block node is the node's): only the left halves are scored.
// Ragged lengths (kv_lens) and a page table are handled per row.
#pragma once
#include "common.h"
#include "launch.h"

namespace hipattn {

// SPLIT = false: one wave per (sequence, head), four independent problems per workgroup.
// SPLIT = true : one workgroup per (sequence, head); the four waves score a quarter of the
//                branches each (stage i goes to wave i % 4), meet at a barrier, run the selection
//                redundantly and write a quarter of the survivors each.  Used up to 8192 problems
//                (see launch_e).
template <int E, int BK, int D, int ROWS, bool PAGED, bool SPLIT>
__global__ __launch_bounds__(kThreads, E == 16 ? 3 : 1) void mask_decode_kernel(KParams p, int xcd_map)
{
    constexpr int NB = 64 * E;
    constexpr int LPR = D / 8;        // lanes per key row
    constexpr int RPW = 64 / LPR;     // rows (= branches) per wave-wide load
    constexpr int U = ROWS / BK;      // branches per lane group and stage: ROWS row loads per lane, two stages in flight
    typedef uint32_t stage_t __attribute__((ext_vector_type(4 * U * BK)));
    constexpr int NW = SPLIT ? 1 : 4;  // private copies of the per-problem LDS state
    constexpr int WS = SPLIT ? 4 : 1;  // waves sharing one problem
    // Two buffers of NB words swap roles every round: one holds the node list (NB/2 starts, then NB/2 ends), the other
    // receives the round's score keys and, once the selection has them in registers, the next node list.
    __shared__ uint32_t buf_s[NW][2][NB];
    __shared__ uint32_t nkey_s[NW][NB / 2];  // score key of the branch that became each node

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // (uniform: what follows from it stays in scalar registers)
    const int grp = lane / LPR, lc = lane % LPR;
    const int own = SPLIT ? 0 : wave;  // which LDS copy
    int64_t wg;
    if (SPLIT) {
        // keep the query heads of a KV group on one XCD (blockIdx.x % 8), next to each other in time
        const int64_t bid = blockIdx.x;
        if (xcd_map) {
            const int64_t seq = bid >> 3, gi = (bid & 7) + 8 * (seq / p.g);
            wg = gi * p.g + seq % p.g;  // = (b * hkv + hk) * g + head in group = b * hq + h
        } else {
            wg = bid;
        }
    } else {
        wg = (int64_t)blockIdx.x * 4 + wave;
    }
    if (wg >= (int64_t)p.batch * p.hq) return;
    const int b = (int)(wg / p.hq), h = (int)(wg % p.hq), hk = h / p.g;
    const int kb = p.kb;
    const int kv_len = p.kv_lens ? p.kv_lens[b] : p.max_kv_len;
    int32_t *out = p.idx_out + wg * kb;

    // BK = key rows scored per block; with a key sampling stride the block itself is bk = BK * b_sk keys
    const int bsk = p.b_sk, bk = BK * bsk;
    const int Tb = kv_len > 0 ? (kv_len + bk - 1) / bk : 0;
    if (Tb <= kb) {
        for (int j = SPLIT ? (int)threadIdx.x : lane; j < kb; j += SPLIT ? kThreads : 64) out[j] = j < Tb ? j * bk : kSentinel;
        return;
    }
    // all waves of a problem hold identical copies of its state when SPLIT
    auto sync_problem = [&]() __attribute__((always_inline)) {
        if (SPLIT) __syncthreads(); else wave_lds_sync();
    };
    const int tix = SPLIT ? (int)threadIdx.x : lane, tn = SPLIT ? kThreads : 64;

    const uint4 qv = *(const uint4 *)((const bf16_t *)p.Q + (int64_t)b * p.qs_b + (int64_t)h * p.qs_h + lc * 8);
    {
        int *ns0 = (int *)buf_s[own][0], *ne0 = ns0 + NB / 2;
        const int a = Tb / kb, r = Tb % kb;
        for (int j = tix; j < kb; j += tn) {
            ns0[j] = chunk_bound(j, a, r, kb);
            ne0[j] = chunk_bound(j + 1, a, r, kb);
        }
    }
    sync_problem();

    const bf16_t *Kbase = (const bf16_t *)p.K;
    const int64_t back_delta = (const bf16_t *)p.Kback - Kbase;  // elements from the resident pool to the backing pool
    int cur = 0;
    bool carry = false;  // a round in which one child of every node keeps the node's score (never the first round)
    // side of a node's children that is scored in a carry round: the left one when the LAST block
    // represents (the right child ends where the node ends), the right one for FIRST
    // (with the centre representative only the final round carries: there every node is one or two blocks long, a
    // one-block node is its own representative and the right half of a two-block node is the node's representative,
    // so the left children alone are scored)
    const int side = p.rep_pos == 1 ? 1 : 0;
    // ensemble sample: the round whose selection compares perturbed scores (-1: none)
    const int ens_round = ens_round_of(p.ens_sample, (Tb + kb - 1) / kb);
    const uint32_t ens_hash = ens_round >= 0 ? ens_unit_hash(p.ens_seed, p.ens_sample, b, h, 0) : 0u;
    int round = 0;
    for (int maxlen = (Tb + kb - 1) / kb; maxlen > 1; maxlen = (maxlen + 1) >> 1, ++round) {
        const int *ns = (const int *)buf_s[own][cur], *ne = ns + NB / 2;
        uint32_t *keys = buf_s[own][cur ^ 1];  // every slot below 2 kb is written by the scoring loop
        uint32_t *nkey = nkey_s[own];
        // work items of the scoring loop: every branch slot, or in a carry round one per node
        const int n_items = carry ? kb : 2 * kb;

        // one stage = U branches per lane group: node lookup, then the (unconditional) loads of
        // the representative block's BK rows.  t0 < 0 marks an empty branch.
        auto fetch = [&](int base, stage_t &kv, int (&t0)[U]) __attribute__((always_inline)) {
            int pg[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int item = base + u * RPW + grp;
                const int slot = carry ? 2 * item + side : item, node = slot >> 1;
                bool ok = node < kb;
                int t = 0;
                if (ok) {
                    const int s = ns[node], e = ne[node];
                    const int mid = s + ((e - s) >> 1);
                    const int bs = (slot & 1) ? mid : s, be = (slot & 1) ? e : mid;
                    ok = be > bs;
                    if (ok) t = rep_block(bs, be, p.rep_pos) * bk;
                }
                t0[u] = ok ? t : -1;
                pg[u] = page_of_row<PAGED>(p, b, ok ? t : 0);  // all page lookups of the stage first
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int t = t0[u] >= 0 ? t0[u] : 0;
                // (a negative page-table entry names a page of the backing pool)
                const bf16_t *src = Kbase + row_offset_bank<PAGED>(p, b, hk, t, pg[u], back_delta) + lc * 8;
#pragma unroll
                for (int n = 0; n < BK; ++n) {
                    // rows past the end of the sequence re-read its last row and are ignored below
                    const int dn = t0[u] >= 0 ? min(n * bsk, kv_len - 1 - t) : 0;
                    const uint4 x = *(const uint4 *)(src + (int64_t)dn * p.ks_r);
                    const int q4 = 4 * (u * BK + n);
                    kv[q4] = x.x; kv[q4 + 1] = x.y; kv[q4 + 2] = x.z; kv[q4 + 3] = x.w;
                }
            }
        };
        auto score = [&](int base, const stage_t &kv, const int (&t0)[U]) __attribute__((always_inline)) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float best = -INFINITY;
#pragma unroll
                for (int n = 0; n < BK; ++n) {
                    const int q4 = 4 * (u * BK + n);
                    const float dsum = row_group_sum<LPR>(dot8_bf16(qv, make_uint4(kv[q4], kv[q4 + 1], kv[q4 + 2], kv[q4 + 3])));
                    if (t0[u] + n * bsk < kv_len) best = fmaxf(best, dsum);
                }
                const int item = base + u * RPW + grp;
                const int slot = carry ? 2 * item + side : item;
                if (lc == 0 && slot < NB) {
                    keys[slot] = t0[u] >= 0 ? score_key(best) : 0u;
                    if (carry) {
                        // the sibling keeps the node's score; a left sibling may be empty (one-block node)
                        const int node = slot >> 1;
                        const bool sib = node < kb && (side == 0 || ne[node] - ns[node] > 1);
                        keys[slot ^ 1] = sib ? nkey[node] : 0u;
                    }
                }
            }
        };

        constexpr int STEP = RPW * U;   // branches per stage
        constexpr int STRIDE = WS * STEP;  // distance between two stages of the same wave
        stage_t ka, kbuf;
        int ta[U], tb[U];
        const int first = SPLIT ? wave * STEP : 0;
        if (first < n_items) fetch(first, ka, ta);
        for (int base = first; base < n_items; base += 2 * STRIDE) {
            const bool has_b = base + STRIDE < n_items;
            if (has_b) fetch(base + STRIDE, kbuf, tb);
            score(base, ka, ta);
            if (has_b) {
                if (base + 2 * STRIDE < n_items) fetch(base + 2 * STRIDE, ka, ta);
                score(base + STRIDE, kbuf, tb);
            }
        }
        sync_problem();

        uint32_t key[E];
#pragma unroll
        for (int i = 0; i < E; ++i) key[i] = i * 64 + lane < 2 * kb ? keys[i * 64 + lane] : 0u;
        if (PAGED && p.touched) {
            // pages read this round: the representative block of every real branch (a branch whose score was
            // carried over had the same block read in an earlier round)
            for (int slot = tix; slot < 2 * kb; slot += tn) {
                if (keys[slot] != 0u) {
                    const int node = slot >> 1;
                    const int s = ns[node], e = ne[node];
                    const int mid = s + ((e - s) >> 1);
                    touch_page(p, b, rep_block((slot & 1) ? mid : s, (slot & 1) ? e : mid, p.rep_pos) * bk);
                }
            }
        }
        // the survivors go where the keys were: every wave of the problem has to hold its copy of them first
        if (SPLIT) __syncthreads();
        bool keep[E];
        int dest[E];
        if (round == ens_round) {
            // the selection sees the perturbed scores; key[] keeps the true ones (they are what a later round carries)
            uint32_t ksel[E];
#pragma unroll
            for (int i = 0; i < E; ++i) {
                ksel[i] = 0u;
                if (key[i] != 0u) {
                    const int slot = i * 64 + lane, node = slot >> 1;
                    const int s = ns[node], e = ne[node];
                    const int mid = s + ((e - s) >> 1);
                    ksel[i] = ens_key(key[i], ens_hash, rep_block((slot & 1) ? mid : s, (slot & 1) ? e : mid, p.rep_pos), p.ens_r);
                }
            }
            select_topk_ordered<E>(ksel, kb, keep, dest);
        } else {
            select_topk_ordered<E>(key, kb, keep, dest);
        }
        int *ns2 = (int *)keys, *ne2 = ns2 + NB / 2;
#pragma unroll
        for (int i = 0; i < E; ++i) {
            if (keep[i] && (!SPLIT || (i & 3) == wave)) {
                const int slot = i * 64 + lane, node = slot >> 1;
                const int s = ns[node], e = ne[node];
                const int mid = s + ((e - s) >> 1);
                ns2[dest[i]] = (slot & 1) ? mid : s;
                ne2[dest[i]] = (slot & 1) ? e : mid;
                nkey[dest[i]] = key[i];
            }
        }
        cur ^= 1;
        carry = p.rep_pos != 0 || ((maxlen + 1) >> 1) == 2;
        sync_problem();
    }

    const int *ns = (const int *)buf_s[own][cur];
    for (int j = tix; j < kb; j += tn) out[j] = ns[j] * bk;
}

template <int BK, int D, int ROWS, bool SPLIT>
static hipError_t launch_r(const KParams &p, dim3 grid, int xcd_map, hipStream_t st)
{
    dim3 block(kThreads);
#define HIPATTN_LAUNCH(EV)                                                                                  \
    do {                                                                                                    \
        if (p.page_table) hipLaunchKernelGGL((mask_decode_kernel<EV, BK, D, ROWS, true, SPLIT>), grid, block, 0, st, p, xcd_map);  \
        else hipLaunchKernelGGL((mask_decode_kernel<EV, BK, D, ROWS, false, SPLIT>), grid, block, 0, st, p, xcd_map);       \
    } while (0)
    if (p.kb <= 128) HIPATTN_LAUNCH(4);
    else if (p.kb <= 256) HIPATTN_LAUNCH(8);
    else if (p.kb <= 512) HIPATTN_LAUNCH(16);
    else HIPATTN_LAUNCH(32);
#undef HIPATTN_LAUNCH
    return hipGetLastError();
}

// Up to 8192 problems: a workgroup per (sequence, head), four waves sharing the scoring, so that enough loads are in
// flight per compute unit and the selection of one problem overlaps with the loads of the others.  Beyond that a wave
// per problem (nothing computed twice, no barriers) is faster.  Measured with 32 query heads over 8 kv heads, k/bk =
// 256, workgroup per problem against wave per problem: 2048 problems -8 %, 4096 -4 %, 8192 -1 to -4 %, 16384 +6 %,
// 32768 +14 %.
template <int BK, int D>
static hipError_t launch_e(const KParams &p, hipStream_t st)
{
    const int64_t problems = (int64_t)p.batch * p.hq;
    if (problems <= 8192) {
        const int64_t groups = (int64_t)p.batch * p.hkv;
        const int xcd_map = groups % 8 == 0 ? 1 : 0;
        return launch_r<BK, D, 8, true>(p, dim3((unsigned)problems), xcd_map, st);
    }
    return launch_r<BK, D, 8, false>(p, dim3((unsigned)((problems + 3) / 4)), 0, st);
}

// One translation unit per (head dim, block width) instantiates this: WIDE = 4 or 8 scored rows per block, else 1 or 2.
template <int D, bool WIDE> hipError_t launch_mask_decode_variant(const KParams &p, hipStream_t st)
{
    if ((int64_t)p.batch * p.hq == 0) return hipSuccess;
    const int rows = p.bk / p.b_sk;
    if constexpr (WIDE) return rows == 4 ? launch_e<4, D>(p, st) : launch_e<8, D>(p, st);
    else return rows == 1 ? launch_e<1, D>(p, st) : launch_e<2, D>(p, st);
}

}  // namespace hipattn
