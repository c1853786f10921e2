// Shape-generic hierarchical mask estimation (paper Alg. 1, block form of Sec. 3.2).
//
// One workgroup (4 waves) per (sequence, query head, query block).  Node and branch
// ranges live in LDS, branch scores are plain fp32 dot products taken by 16-lane groups
// (one key row per group per step), the per-round top-k is the ordered threshold
// selection of common.h.  Any bq <= 64, bk <= 16, k/bk <= 1024, contiguous or paged K,
// prefill or decode.  The tuned kernels (mask_mfma.hip, mask_decode.hip) cover the
// benchmark shapes; this one covers everything else and serves fp32.
#include "common.h"
#include "launch.h"

namespace hipattn {

template <typename T, int D, int E>
__global__ __launch_bounds__(kThreads) void mask_generic_kernel(KParams p)
{
    constexpr int NB = 64 * E;   // branch slots (two per node)
    constexpr int CH = D / 16;   // channels per lane of a 16-lane group
    extern __shared__ float q_s[];  // [bq][D]
    __shared__ int nd_s[NB / 2], nd_e[NB / 2];
    __shared__ int br_s[NB], br_e[NB];
    __shared__ uint32_t keys[NB];

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
    const int L = min(kv_len, pos0 + n_rows);  // visible prefix of this query block
    int32_t *out = p.idx_out + unit * kb;

    const int Tb = L > 0 ? (L + bk - 1) / bk : 0;
    if (Tb <= kb) {  // nothing to prune: every visible block is selected
        for (int j = tid; j < kb; j += kThreads) out[j] = j < Tb ? j * bk : kSentinel;
        return;
    }

    const T *Qb = (const T *)p.Q + (int64_t)b * p.qs_b + (int64_t)h * p.qs_h + (int64_t)row0 * p.qs_r;
    for (int i = tid; i < n_rows * D; i += kThreads) q_s[i] = ld_f32(Qb + (int64_t)(i / D) * p.qs_r + (i % D));

    // initial nodes: kb chunks of [0, Tb) with rounded bounds; all non-empty because Tb > kb
    const int a = Tb / kb, r = Tb % kb;
    for (int j = tid; j < kb; j += kThreads) {
        nd_s[j] = chunk_bound(j, a, r, kb);
        nd_e[j] = chunk_bound(j + 1, a, r, kb);
    }
    __syncthreads();

    const T *Kbase = (const T *)p.K, *Kback = (const T *)p.Kback;
    const int grp = tid >> 4, l16 = tid & 15;

    // ensemble sample: the round whose selection compares perturbed scores (-1: none)
    const int ens_round = ens_round_of(p.ens_sample, a + (r ? 1 : 0));
    const uint32_t ens_hash = ens_round >= 0 ? ens_unit_hash(p.ens_seed, p.ens_sample, b, h, qb) : 0u;
    int round = 0;
    // maxlen bounds the longest node; one more round than strictly needed is a no-op
    for (int maxlen = a + (r ? 1 : 0); maxlen > 1; maxlen = (maxlen + 1) >> 1, ++round) {
        // split every node into its left and right branch (slot 2j, 2j+1); left may be empty
        for (int j = tid; j < NB / 2; j += kThreads) {
            int s = 0, mid = 0, e = 0;
            if (j < kb) { s = nd_s[j]; e = nd_e[j]; mid = s + ((e - s) >> 1); }
            br_s[2 * j] = s; br_e[2 * j] = mid;
            br_s[2 * j + 1] = mid; br_e[2 * j + 1] = e;
            // a real branch starts at "-inf" (it may end up without an admissible pair), an empty one at 0
            keys[2 * j] = mid > s ? kKeyNegInf : 0u;
            keys[2 * j + 1] = e > mid ? kKeyNegInf : 0u;
        }
        __syncthreads();

        // score: one key row of a representative block per 16-lane group and step
        const int n_key_rows = 2 * kb * bk;
        for (int rr = grp; rr < n_key_rows; rr += kThreads / 16) {
            const int slot = rr / bk, n = rr - slot * bk;
            if (n % p.b_sk) continue;  // key sampling stride
            const int s = br_s[slot], e = br_e[slot];
            if (e <= s) continue;
            const int t = rep_block(s, e, p.rep_pos) * bk + n;  // key of the representative block
            if (t >= kv_len) continue;
            bool miss;
            const int64_t off = kv_row_offset(p, b, hk, t, miss);
            const T *krow = (miss ? Kback : Kbase) + off + l16 * CH;
            if (p.touched && l16 == 0) touch_page(p, b, t);
            float kreg[CH];
#pragma unroll
            for (int c = 0; c < CH; ++c) kreg[c] = ld_f32(krow + c);
            float best = -INFINITY;
            for (int m = 0; m < n_rows; m += p.b_sq) {  // row sampling stride
                if (t > pos0 + m) continue;  // causal: key in the future of this row
                const float *qrow = q_s + m * D + l16 * CH;
                float acc = 0.f;
#pragma unroll
                for (int c = 0; c < CH; ++c) acc = fmaf(qrow[c], kreg[c], acc);
                acc += __shfl_xor(acc, 8, 16);
                acc += __shfl_xor(acc, 4, 16);
                acc += __shfl_xor(acc, 2, 16);
                acc += __shfl_xor(acc, 1, 16);
                best = fmaxf(best, acc);
            }
            if (l16 == 0 && best > -INFINITY) atomicMax(&keys[slot], score_key(best));
        }
        __syncthreads();

        // every wave selects redundantly; wave (i % 4) writes the survivors of register i
        uint32_t key[E];
        bool keep[E];
        int dest[E];
#pragma unroll
        for (int i = 0; i < E; ++i) {
            key[i] = keys[i * 64 + lane];
            if (round == ens_round && key[i] != 0u)
                key[i] = ens_key(key[i], ens_hash, rep_block(br_s[i * 64 + lane], br_e[i * 64 + lane], p.rep_pos), p.ens_r);
        }
        select_topk_ordered<E>(key, kb, keep, dest);
#pragma unroll
        for (int i = 0; i < E; ++i) {
            if ((i & 3) == wave && keep[i]) {
                nd_s[dest[i]] = br_s[i * 64 + lane];
                nd_e[dest[i]] = br_e[i * 64 + lane];
            }
        }
        __syncthreads();
    }

    for (int j = tid; j < kb; j += kThreads) out[j] = nd_s[j] * bk;
}

template <typename T, int D>
static hipError_t launch_de(const KParams &p, int64_t units, size_t smem, hipStream_t st)
{
    dim3 grid((unsigned)units), block(kThreads);
    if (p.kb <= 64) hipLaunchKernelGGL((mask_generic_kernel<T, D, 2>), grid, block, smem, st, p);
    else if (p.kb <= 256) hipLaunchKernelGGL((mask_generic_kernel<T, D, 8>), grid, block, smem, st, p);
    else if (p.kb <= 512) hipLaunchKernelGGL((mask_generic_kernel<T, D, 16>), grid, block, smem, st, p);
    else hipLaunchKernelGGL((mask_generic_kernel<T, D, 32>), grid, block, smem, st, p);
    return hipGetLastError();
}

hipError_t launch_mask_generic(const KParams &p, bool bf16, hipStream_t st)
{
    const int64_t units = (int64_t)p.batch * p.hq * p.nqb;
    if (units == 0) return hipSuccess;
    const size_t smem = (size_t)p.bq * p.d * sizeof(float);
    if (bf16) return p.d == 64 ? launch_de<bf16_t, 64>(p, units, smem, st) : launch_de<bf16_t, 128>(p, units, smem, st);
    return p.d == 64 ? launch_de<float, 64>(p, units, smem, st) : launch_de<float, 128>(p, units, smem, st);
}

}  // namespace hipattn
