// Hierarchical mask estimation for bf16 prefill on CDNA4 matrix cores
// (paper Alg. 1; the block approximation of Sec. 3.2 is what makes the branch scoring a
// dense query-block x gathered-key-rows contraction).
//
// One workgroup of 4 waves per (sequence, query head, query block).
//   * The query block (<= 64 rows) sits in registers of every wave as the MFMA A operand.
//   * A round scores 2*kb branches = 2*kb*bk gathered key rows in tiles of 32 rows; tile i
//     goes to wave i % 4.  Every lane loads its own key row straight from global memory in
//     the B-operand layout (lane l: row l % 32, 16-byte chunk l / 32 of each 32-byte step),
//     the next tile's loads are in flight while the current one is multiplied.
//   * v_mfma_f32_32x32x16_bf16 gives a 32(query) x 32(key) score tile; the branch score is
//     the max over the admissible query rows (in-lane, then lanes l and l+32) and over the
//     bk keys of the block (neighbouring lanes).
//   * Scores go to LDS as order-preserving integer keys; after ONE barrier every wave runs
//     the ordered threshold selection redundantly and writes the surviving nodes into its
//     own private node list, so no second barrier is needed.
// Node ranges are block indices [s, e); the list stays sorted by position throughout, which
// is why the result needs no sort.
#include "common.h"
#include "launch.h"

namespace hipattn {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

// (sequence, head, query block) of a workgroup.  With `xcd_map` the grid is laid out so that
// the workgroups an XCD receives (blockIdx.x % 8) all read the same KV head, walk the query
// blocks from the longest prefix down, and keep the query heads of a KV group adjacent.
__device__ __forceinline__ bool decode_unit(const KParams &p, int xcd_map, int &b, int &h, int &qb)
{
    const int64_t bid = blockIdx.x;
    const int per_group = p.g * p.nqb;
    int64_t group, within;
    if (xcd_map) {
        const int xcd = (int)(bid & 7);
        const int64_t seq = bid >> 3;
        group = xcd + 8 * (seq / per_group);
        within = seq % per_group;
        if (group >= (int64_t)p.batch * p.hkv) return false;
    } else {
        group = bid / per_group;
        within = bid % per_group;
    }
    qb = p.nqb - 1 - (int)(within / p.g);
    h = (int)(group % p.hkv) * p.g + (int)(within % p.g);
    b = (int)(group / p.hkv);
    return true;
}

template <int MT, int E, int D>
__global__ __launch_bounds__(kThreads) void mask_mfma_kernel(KParams p, int log_bk, int xcd_map)
{
    constexpr int NB = 64 * E;  // branch slots
    constexpr int KS = D / 16;  // MFMA k-steps per key row
    __shared__ uint32_t keys[2][NB];
    __shared__ int nds[4][2][NB / 2], nde[4][2][NB / 2];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, hh = lane >> 5;
    int b, h, qb;
    if (!decode_unit(p, xcd_map, b, h, qb)) return;
    const int hk = h / p.g;
    const int kb = p.kb, bk = 1 << log_bk;

    const int kv_len = p.kv_lens ? p.kv_lens[b] : p.max_kv_len;
    const int row0 = qb * p.bq;
    const int n_rows = min(p.bq, p.q_len - row0);
    const int pos0 = kv_len - p.q_len + row0;
    const int L = min(kv_len, pos0 + n_rows);
    int32_t *out = p.idx_out + (((int64_t)b * p.hq + h) * p.nqb + qb) * kb;

    const int Tb = L > 0 ? (L + bk - 1) >> log_bk : 0;
    if (Tb <= kb) {
        for (int j = tid; j < kb; j += kThreads) out[j] = j < Tb ? j << log_bk : kSentinel;
        return;
    }

    // query block as MFMA A operand: lane holds row (lane % 32) [+32], 8 channels per k-step
    bf16x8 qf[MT][KS];
    {
        const bf16_t *Qb = (const bf16_t *)p.Q + (int64_t)b * p.qs_b + (int64_t)h * p.qs_h + (int64_t)row0 * p.qs_r;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int i = mt * 32 + col;
#pragma unroll
            for (int kk = 0; kk < KS; ++kk) {
                uint4 v = make_uint4(0, 0, 0, 0);
                if (i < n_rows) v = *(const uint4 *)(Qb + (int64_t)i * p.qs_r + kk * 16 + hh * 8);
                qf[mt][kk] = __builtin_bit_cast(bf16x8, v);
            }
        }
    }

    for (int i = tid; i < 2 * NB; i += kThreads) (&keys[0][0])[i] = 0;
    {
        const int a = Tb / kb, r = Tb % kb;
        for (int j = lane; j < kb; j += 64) {
            nds[wave][0][j] = chunk_bound(j, a, r, kb);
            nde[wave][0][j] = chunk_bound(j + 1, a, r, kb);
        }
    }
    __syncthreads();

    const bf16_t *Kbase = (const bf16_t *)p.K;
    const int n_tiles = (2 * kb * bk + 31) >> 5;
    const bool full_rows = n_rows == 32 * MT;
    int cur = 0, round = 0;

    for (int maxlen = (Tb + kb - 1) / kb; maxlen > 1; maxlen = (maxlen + 1) >> 1, ++round) {
        const int *ns = nds[wave][cur], *ne = nde[wave][cur];
        uint32_t *kout = keys[round & 1];

        // metadata + loads of one tile of 32 gathered key rows
        auto fetch = [&](int tile, uint4(&kr)[KS], int &t, int &slot, bool &slot_ok, bool &row_ok) {
            const int rr = tile * 32 + col;
            slot = rr >> log_bk;
            const int node = slot >> 1;
            slot_ok = node < kb;
            t = 0;
            if (slot_ok) {
                const int s = ns[node], e = ne[node];
                const int mid = s + ((e - s) >> 1);
                const int bs = (slot & 1) ? mid : s, be = (slot & 1) ? e : mid;
                slot_ok = be > bs;
                t = ((bs + ((be - bs) >> 1)) << log_bk) + (rr & (bk - 1));
            }
            row_ok = slot_ok && t < kv_len;
            if (row_ok) {
                const bf16_t *src = Kbase + kv_row_offset(p, b, hk, t) + hh * 8;
#pragma unroll
                for (int kk = 0; kk < KS; ++kk) kr[kk] = *(const uint4 *)(src + kk * 16);
            } else {
#pragma unroll
                for (int kk = 0; kk < KS; ++kk) kr[kk] = make_uint4(0, 0, 0, 0);
            }
        };

        uint4 kc[KS], kn[KS];
        int t_c, slot_c, t_n = 0, slot_n = 0;
        bool sok_c, rok_c, sok_n = false, rok_n = false;
        int tile = wave;
        if (tile < n_tiles) fetch(tile, kc, t_c, slot_c, sok_c, rok_c);
        for (; tile < n_tiles; tile += 4) {
            const bool has_next = tile + 4 < n_tiles;
            if (has_next) fetch(tile + 4, kn, t_n, slot_n, sok_n, rok_n);

            f32x16 acc[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mt][r] = 0.f;
#pragma unroll
            for (int kk = 0; kk < KS; ++kk)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[mt][kk], __builtin_bit_cast(bf16x8, kc[kk]),
                                                                      acc[mt], 0, 0, 0);
            // max over the admissible query rows of this lane's key column
            const int lo = t_c - pos0;  // rows i < lo would look into the future
            float v = -INFINITY;
            if (full_rows && __ballot(rok_c && lo > 0) == 0) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) v = fmaxf(v, acc[mt][r]);
            } else {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int i = mt * 32 + (r >> 2) * 8 + hh * 4 + (r & 3);
                        if (i >= lo && i < n_rows) v = fmaxf(v, acc[mt][r]);
                    }
            }
            if (!rok_c) v = -INFINITY;
            v = fmaxf(v, __shfl_xor(v, 32, 64));
            for (int o = 1; o < bk; o <<= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
            if (hh == 0 && (col & (bk - 1)) == 0 && slot_c < NB) kout[slot_c] = sok_c ? score_key(v) : 0u;

            if (has_next) {
#pragma unroll
                for (int kk = 0; kk < KS; ++kk) kc[kk] = kn[kk];
                t_c = t_n; slot_c = slot_n; sok_c = sok_n; rok_c = rok_n;
            }
        }
        __syncthreads();

        // selection, redundantly per wave, into this wave's private next node list
        uint32_t key[E];
        bool keep[E];
        int dest[E];
#pragma unroll
        for (int i = 0; i < E; ++i) key[i] = kout[i * 64 + lane];
        select_topk_ordered<E>(key, kb, keep, dest);
        int *ns2 = nds[wave][cur ^ 1], *ne2 = nde[wave][cur ^ 1];
#pragma unroll
        for (int i = 0; i < E; ++i) {
            if (keep[i]) {
                const int slot = i * 64 + lane, node = slot >> 1;
                const int s = ns[node], e = ne[node];
                const int mid = s + ((e - s) >> 1);
                ns2[dest[i]] = (slot & 1) ? mid : s;
                ne2[dest[i]] = (slot & 1) ? e : mid;
            }
        }
        cur ^= 1;
        wave_lds_sync();
    }

    if (wave == 0) {
        const int *ns = nds[0][cur];
        for (int j = lane; j < kb; j += 64) out[j] = ns[j] << log_bk;
    }
}

template <int MT, int D>
static hipError_t launch_e(const KParams &p, int log_bk, int xcd_map, dim3 grid, hipStream_t st)
{
    dim3 block(kThreads);
    if (p.kb <= 128) hipLaunchKernelGGL((mask_mfma_kernel<MT, 4, D>), grid, block, 0, st, p, log_bk, xcd_map);
    else if (p.kb <= 256) hipLaunchKernelGGL((mask_mfma_kernel<MT, 8, D>), grid, block, 0, st, p, log_bk, xcd_map);
    else hipLaunchKernelGGL((mask_mfma_kernel<MT, 16, D>), grid, block, 0, st, p, log_bk, xcd_map);
    return hipGetLastError();
}

bool mask_mfma_supported(const KParams &p, bool bf16)
{
    // k/bk above 512 would need more than the 64 KB of statically allocated LDS: generic kernel
    return bf16 && p.q_len > 1 && p.bk <= 16 && (p.bk & (p.bk - 1)) == 0 && p.bq <= 64 && p.kb <= 512;
}

hipError_t launch_mask_mfma(const KParams &p, hipStream_t st)
{
    int log_bk = 0;
    while ((1 << log_bk) < p.bk) ++log_bk;
    const int64_t groups = (int64_t)p.batch * p.hkv;
    const int64_t per_group = (int64_t)p.g * p.nqb;
    const int xcd_map = groups % 8 == 0 ? 1 : 0;
    const int64_t units = groups * per_group;
    if (units == 0) return hipSuccess;
    dim3 grid((unsigned)units);
    if (p.bq <= 32) return p.d == 64 ? launch_e<1, 64>(p, log_bk, xcd_map, grid, st) : launch_e<1, 128>(p, log_bk, xcd_map, grid, st);
    return p.d == 64 ? launch_e<2, 64>(p, log_bk, xcd_map, grid, st) : launch_e<2, 128>(p, log_bk, xcd_map, grid, st);
}

}  // namespace hipattn
