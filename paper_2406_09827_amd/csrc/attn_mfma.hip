// Block-sparse attention for bf16 prefill on CDNA4 matrix cores (paper Eq. 2-3; the
// "block sparse flash attention" of the appendix: online softmax over the gathered keys).
//
// Work item = one wave = one (sequence, query head, query block, 32-row query tile); four
// independent work items per workgroup, no workgroup barrier anywhere.
// Per tile of 32 gathered keys:
//   S^T = K_tile . Q^T     v_mfma_f32_32x32x16_bf16, A = key rows (loaded coalesced, staged in a
//                          swizzled LDS tile, read back one row per lane), B = the query tile
//                          held in registers.
//                          The result has one query per lane and 16 keys in its registers,
//                          so the softmax statistics of a query are lane-local (plus one
//                          exchange with lane ^ 32) and P^T is already in B-operand layout.
//   O^T += V_tile^T . P^T  (P as hi + lo bf16 terms) the value rows are loaded coalesced, staged
//                          in this wave's LDS slice and read back channel-major with the LDS
//                          transpose read ds_read_b64_tr_b16 (the contraction runs over keys, so
//                          V has to be transposed on the way to the A operand).
// The key positions of a tile and their row offsets are published through a small per-wave
// LDS array so that every lane can mask by (key position, query position).
#include "common.h"
#include "launch.h"

namespace hipattn {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((address_space(3))) s16x4 *lds_s16x4_ptr;

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    f32x2 x = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
}

// MODE 0: contiguous K/V, a (sequence, kv head) slice below 4 GB: rows are addressed by a scalar slice base
//         plus a 32-bit lane offset (one shift-add per row instead of 64-bit vector arithmetic);
// MODE 1: paged pool; MODE 2: contiguous, any size (64-bit row addresses).
// SPLIT: the workgroup takes ONE work item; wave w walks key tiles w, w + 4, ... with its own softmax state and the
//        four states are merged through LDS at the end (for launches with too few work items to fill the GPU).
template <int D, int MODE, bool SPLIT>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2))) void attn_mfma_kernel(KParams p, int log_bk, int mtn, int xcd_map)
{
    constexpr bool PAGED = MODE == 1, A32 = MODE == 0;
    constexpr int KS = D / 16;     // k-steps of S^T = K Q^T
    constexpr int CT = D / 32;     // 32-channel tiles of O^T
    constexpr int PITCH = D + 32;  // value tile row pitch in bf16: 64 bytes of padding per row (4 keys x 2 channel halves fill the 64 banks)
    constexpr int CPR = D / 8;     // 16-byte chunks per row
    constexpr int RPI = 64 / CPR;  // rows covered by one wave-wide 16-byte load
    constexpr int NLD = 32 / RPI;  // such loads per 32-row tile
    constexpr int ROWB = D * 2;    // bytes per key row in the (swizzled, unpadded) key tile
    typedef uint32_t stage_t __attribute__((ext_vector_type(4 * NLD)));
    __shared__ __attribute__((aligned(16))) bf16_t vt_s[4][32 * PITCH];
    __shared__ __attribute__((aligned(16))) uint4 kt_s[4][32 * ROWB / 16];
    __shared__ __attribute__((aligned(16))) int tk_s[4][2][32];
    __shared__ __attribute__((aligned(16))) uint32_t mo_s[4][32];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, hh = lane >> 5;
    const int lg = lane / CPR, lc = lane % CPR;  // loading role: rows lg*NLD .. +NLD-1, chunk lc

    // ---- which (sequence, head, query block, query tile) this wave owns
    const uint32_t groups = (uint32_t)p.batch * (uint32_t)p.hkv;
    const uint32_t per_group = (uint32_t)p.g * (uint32_t)p.nqb * (uint32_t)mtn;
    uint32_t group, o;
    if (!place_item(xcd_map, blockIdx.x, SPLIT ? 1 : 4, SPLIT ? 0 : wave, per_group, groups, group, o)) return;
    const uint32_t gm = (uint32_t)(p.g * mtn), oq = o / gm, rem = o - oq * gm;
    const int qb = p.nqb - 1 - (int)oq;
    const int b = (int)(group / (uint32_t)p.hkv), hk = (int)(group - (uint32_t)b * (uint32_t)p.hkv);
    const int h = hk * p.g + (mtn == 2 ? (int)(rem >> 1) : (int)rem), mt = mtn == 2 ? (int)(rem & 1) : 0;

    const int kv_len = p.kv_lens ? p.kv_lens[b] : p.max_kv_len;
    const int row0 = qb * p.bq + mt * 32;
    const int n_rows = min(32, min(p.bq, p.q_len - qb * p.bq) - mt * 32);
    if (n_rows <= 0) return;
    const int pos0 = kv_len - p.q_len + row0;  // position of this tile's first query row
    const int32_t *idx = p.idx_in + (((int64_t)b * p.hq + h) * p.nqb + qb) * p.kb;
    const int bk = 1 << log_bk;
    // Key tiles: first the selected blocks, then the sink keys [0, ns), then the window keys
    // [wlo, vis_last).  For a row at position q with vis = min(q+1, kv_len) and
    // w0 = max(vis - n_window, 0): a selected or sink key t counts iff t < w0 (selected also
    // t >= n_sink), a window key iff w0 <= t < vis - so every key counts once.
    const int n_keys = p.kb << log_bk;
    const int vis_last = min(pos0 + n_rows, kv_len);                     // keys any row of the tile may see
    const int wlo = max(min(pos0 + 1, kv_len) - p.n_window, 0);          // window start of the first row
    const int ns = min(p.n_sink, max(vis_last - p.n_window, 0));         // sink keys some row takes as sink
    const int nw = p.n_window > 0 ? max(vis_last - wlo, 0) : 0;
    const int tiles_sel = (n_keys + 31) >> 5, tiles_sink = (ns + 31) >> 5, tiles_win = (nw + 31) >> 5;
    const int n_tiles = tiles_sel + tiles_sink + tiles_win;
    const int w0_first = wlo;                                             // smallest w0 over the rows
    const int w0_last = max(vis_last - p.n_window, 0);                    // largest w0 over the rows

    // ---- query tile as B operand (lane: query col, channels kk*16 + hh*8 ..)
    bf16x8 qf[KS];
    {
        const bf16_t *Qb = (const bf16_t *)p.Q + (int64_t)b * p.qs_b + (int64_t)h * p.qs_h + (int64_t)row0 * p.qs_r;
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (col < n_rows) v = *(const uint4 *)(Qb + (int64_t)col * p.qs_r + kk * 16 + hh * 8);
            qf[kk] = __builtin_bit_cast(bf16x8, v);
        }
    }

    const bf16_t *Kbase = (const bf16_t *)p.K, *Vbase = (const bf16_t *)p.V;
    const int64_t seq_off = (int64_t)b * p.ks_b + (int64_t)hk * p.ks_h;  // contiguous layout: row 0 of this slice
    // the same in every lane: as a scalar (readfirstlane) it becomes the scalar base of the row loads
    const int64_t slice_u = ((int64_t)__builtin_amdgcn_readfirstlane((int)((seq_off * 2) >> 32)) << 32) |
                            (uint32_t)__builtin_amdgcn_readfirstlane((int)(seq_off * 2));
    const char *Kseq = (const char *)p.K + slice_u, *Vseq = (const char *)p.V + slice_u;
    bf16_t *vt = vt_s[wave];
    char *kt = (char *)kt_s[wave];
    uint32_t *mo = mo_s[wave];

    const float c = p.sm_scale * 1.44269504088896340736f;  // scores are kept in log2 units
    constexpr float kSlack = 8.f;
    float m_run = -INFINITY, l_run = 0.f;
    f32x16 oacc[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[ct][r] = 0.f;

    // One tile of 32 gathered keys: lane `col` works out key row col (position or -1, row
    // offset in 16-byte units), publishes both, then every lane loads its share of the key and
    // value rows coalesced.  Rows that do not count load row 0 of the sequence (always mapped,
    // finite) and get probability 0.  Returns flags: bit 0 = some key may count for some row,
    // bit 1 = some (key, row) pair needs masking, bit 2 = window tile.
    // The index entry lane `col` needs for a tile of selected blocks is loaded one tile before fetch()
    // uses it, so that the row loads do not queue behind the latency of the index load.
    auto index_entry = [&](int tile) __attribute__((always_inline)) {
        const int ki = tile * 32 + col;
        return (tile < tiles_sel && ki < n_keys) ? idx[ki >> log_bk] : -1;
    };
    auto fetch = [&](int tile, int first, stage_t &RK, stage_t &RV, int *tk) __attribute__((always_inline)) {
        int t_c = -1;
        int flags;
        if (tile < tiles_sel) {
            const int ki = tile * 32 + col;
            if (ki < n_keys) {
                const int t = first + (ki & (bk - 1));
                if (first >= 0 && first < kv_len && t < kv_len && t >= p.n_sink) t_c = t;
            }
            flags = (__ballot(t_c >= 0 && t_c < w0_last) != 0 ? 1 : 0) | (__ballot(t_c < 0 || t_c >= w0_first) != 0 ? 2 : 0);
        } else if (tile < tiles_sel + tiles_sink) {
            const int t = (tile - tiles_sel) * 32 + col;
            if (t < ns) t_c = t;
            flags = 1 | 2;
        } else {
            const int t = wlo + (tile - tiles_sel - tiles_sink) * 32 + col;
            if (t < vis_last) t_c = t;
            flags = 1 | 2 | 4;  // bit 2: window tile (keys count for the rows whose window holds them)
        }
        {
            const int tr = t_c >= 0 ? t_c : 0;
            // what a loading lane needs to find the row: the page (paged pool) or the row's offset
            // from the start of this sequence / kv head slice in 16-byte units (contiguous)
            const uint32_t m = PAGED ? (uint32_t)page_of_row<true>(p, b, tr)
                                     : (uint32_t)(((int64_t)tr * p.ks_r) >> 3);
            if (hh == 0) {
                tk[col] = t_c;
                mo[col] = m;
            }
        }
        wave_lds_sync();
        uint32_t off[NLD];
#pragma unroll
        for (int j = 0; j < NLD; j += 4) {
            const uint4 m4 = *(const uint4 *)(mo + lg * NLD + j);
            off[j] = m4.x; off[j + 1] = m4.y; off[j + 2] = m4.z; off[j + 3] = m4.w;
        }
        int tkl[NLD];  // positions of this lane's rows (paged variant: the offset inside the page)
        if (PAGED) {
#pragma unroll
            for (int j = 0; j < NLD; j += 4) {
                const int4 t4 = *(const int4 *)(tk + lg * NLD + j);
                tkl[j] = t4.x; tkl[j + 1] = t4.y; tkl[j + 2] = t4.z; tkl[j + 3] = t4.w;
            }
        }
        wave_lds_sync();
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
            int64_t eo;
            const bf16_t *Kp = Kbase, *Vp = Vbase;
            if (PAGED) {
                const int tr = max(tkl[j], 0);
                // (a negative page-table entry names a page of the backing pools)
                eo = row_offset_in<true>(p, b, hk, tr, page_in_pool((int)off[j])) + lc * 8;
                Kp = (const bf16_t *)pool_of((int)off[j], Kbase, p.Kback);
                Vp = (const bf16_t *)pool_of((int)off[j], Vbase, p.Vback);
            } else {
                eo = seq_off + ((int64_t)off[j] << 3) + lc * 8;
            }
            uint4 x, y;
            if (A32) {
                const uint32_t vo = (off[j] << 4) + (uint32_t)lc * 16u;
                x = *(const uint4 *)(Kseq + vo);
                y = *(const uint4 *)(Vseq + vo);
            } else {
                x = *(const uint4 *)(Kp + eo);
                y = *(const uint4 *)(Vp + eo);
            }
            RK[4 * j] = x.x; RK[4 * j + 1] = x.y; RK[4 * j + 2] = x.z; RK[4 * j + 3] = x.w;
            RV[4 * j] = y.x; RV[4 * j + 1] = y.y; RV[4 * j + 2] = y.z; RV[4 * j + 3] = y.w;
        }
        return flags;
    };

    // this wave's tiles: all of them, or every fourth one (SPLIT)
    const int nt = SPLIT ? (n_tiles > wave ? (n_tiles - wave + 3) >> 2 : 0) : n_tiles;
    auto tile_of = [&](int i) __attribute__((always_inline)) { return SPLIT ? wave + 4 * i : i; };
    stage_t RK, RV;
    int flags_next = 0, first_next = -1;
    if (nt > 0) {
        flags_next = fetch(tile_of(0), index_entry(tile_of(0)), RK, RV, tk_s[wave][0]);
        first_next = index_entry(tile_of(1));
    }
    for (int tile = 0; tile < nt; ++tile) {
        const int flags = flags_next;
        const int *tk = tk_s[wave][tile & 1];
        // registers -> LDS: key tile swizzled (chunk lc of row r at slot lc ^ (r % CPR)), value tile padded
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
            const int r = lg * NLD + j;
            *(uint4 *)(kt + r * ROWB + ((lc ^ (r & (CPR - 1))) << 4)) = make_uint4(RK[4 * j], RK[4 * j + 1], RK[4 * j + 2], RK[4 * j + 3]);
            *(uint4 *)(vt + r * PITCH + lc * 8) = make_uint4(RV[4 * j], RV[4 * j + 1], RV[4 * j + 2], RV[4 * j + 3]);
        }
        if (tile + 1 < nt) {
            flags_next = fetch(tile_of(tile + 1), first_next, RK, RV, tk_s[wave][(tile + 1) & 1]);
            first_next = index_entry(tile_of(tile + 2));
        }
        wave_lds_sync();

        if (flags & 1) {
            // ---- S^T = K Q^T: A = key rows from the LDS tile (lane: key row col), B = queries.  All operand reads
            // are issued before the first multiply (one LDS latency per tile, not one per k-step); the wave
            // raises its priority while it feeds the matrix pipe, so that of two waves on a SIMD one multiplies
            // while the other runs its softmax arithmetic instead of both queueing on the same unit.
            f32x16 sacc;
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
            uint4 kv[KS];
#pragma unroll
            for (int kk = 0; kk < KS; ++kk)
                kv[kk] = *(const uint4 *)(kt + col * ROWB + (((kk * 2 + hh) ^ (col & (CPR - 1))) << 4));
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_setprio(2);
#pragma unroll
            for (int kk = 0; kk < KS; ++kk)
                sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kv[kk]), qf[kk], sacc, 0, 0, 0);
            __builtin_amdgcn_s_setprio(0);

            // ---- online softmax for query `col` (both half-waves hold the same query)
            float s[16], mx = -INFINITY;
            if (flags & 2) {
                // positions of the 16 keys this lane holds scores for: rows 8g + 4hh + {0..3};
                // admissible range [lo, hi) of key positions for this lane's query
                const int visq = min(pos0 + col + 1, kv_len);
                const int w0q = max(visq - p.n_window, 0);
                const int lo = (flags & 4) ? w0q : 0, hi = (flags & 4) ? visq : w0q;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int4 tq = *(const int4 *)(tk + 8 * g + 4 * hh);
                    const int tkey[4] = {tq.x, tq.y, tq.z, tq.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const bool ok = tkey[e] >= lo && tkey[e] < hi;
                        s[4 * g + e] = ok ? sacc[4 * g + e] : -INFINITY;
                    }
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) s[r] = sacc[r];
            }
            // raw scores here; the scale (c > 0) is applied to the maximum and inside the exponent
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[r]);
            {   // other half of the query's keys: lane ^ 32
                const unsigned u = __float_as_uint(mx);
                auto sw = __builtin_amdgcn_permlane32_swap(u, u, false, false);
                mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1])) * c;
            }
            // The running reference m_run only has to bound the exponents, it need not be the exact
            // maximum: it moves (and the accumulators are rescaled) only when a tile's maximum exceeds
            // it by more than kSlack (log2 units; probabilities then stay below 2^kSlack, far inside
            // the range of fp32 sums and bf16 operands).  The final division by l cancels the reference.
            const float m_new = mx > m_run + kSlack ? mx : m_run;
            const float m_safe = m_new == -INFINITY ? 0.f : m_new;
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);
#pragma unroll
            for (int r = 0; r < 16; ++r) s[r] = __builtin_amdgcn_exp2f(fmaf(s[r], c, -m_safe));
            // P^T as B operand of the two 16-key steps (registers 8*st .. 8*st+7), rounded to bf16.  The row sum l
            // is taken over the ROUNDED probabilities (v_dot2_f32_bf16 against ones, fp32 accumulation), so that
            // numerator and denominator of the output carry the same weights: the rounding of P then perturbs the
            // weights of a weighted mean by 2^-9 relative instead of adding an error of that size to the output.
            bf16x8 pb[2];
            float lsum = 0.f;
            {
                const bf16x2 ones = __builtin_bit_cast(bf16x2, 0x3f803f80u);
#pragma unroll
                for (int st = 0; st < 2; ++st) {
                    uint32_t hi[4];
#pragma unroll
                    for (int e2 = 0; e2 < 4; ++e2) {
                        hi[e2] = pack_bf16(s[8 * st + 2 * e2], s[8 * st + 2 * e2 + 1]);
                        lsum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, hi[e2]), ones, lsum, false);
                    }
                    pb[st] = __builtin_bit_cast(bf16x8, make_uint4(hi[0], hi[1], hi[2], hi[3]));
                }
            }
            l_run = l_run * alpha + lsum;
            m_run = m_new;
            if (__ballot(alpha != 1.f) != 0) {
#pragma unroll
                for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[ct][r] *= alpha;
            }

            // ---- O^T += V^T P^T: value tile read back channel-major with the LDS transpose read.
            // ds_read_b64_tr_b16 works on blocks of 16 lanes: lanes 4e .. 4e+3 of a block point at 16
            // consecutive bf16 of source row e (e = 0..3), and lane i of the block receives element i
            // of each of the four rows.  Block = (channel half cb, key half hh): rows are 4 consecutive
            // keys, so a lane ends up with 4 keys of its channel - half an A operand per read.
            {
                const int i16 = lane & 15, cb = (lane >> 4) & 1;
                const bf16_t *src0 = vt + (4 * hh + (i16 >> 2)) * PITCH + cb * 16 + (i16 & 3) * 4;
#pragma unroll
                for (int st = 0; st < 2; ++st) {
                    bf16x8 va[CT];
#pragma unroll
                    for (int ct = 0; ct < CT; ++ct) {
                        // keys 16st + 4hh + {0..3} and 16st + 8 + 4hh + {0..3}, channel ct*32 + col
                        const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(src0 + (16 * st) * PITCH + ct * 32));
                        const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(src0 + (16 * st + 8) * PITCH + ct * 32));
                        const uint2 a = __builtin_bit_cast(uint2, lo4), c2 = __builtin_bit_cast(uint2, hi4);
                        va[ct] = __builtin_bit_cast(bf16x8, make_uint4(a.x, a.y, c2.x, c2.y));
                    }
                    // the CT accumulators are independent: interleave them so that no multiply waits
                    // for the one before it
                    __builtin_amdgcn_s_setprio(2);
#pragma unroll
                    for (int ct = 0; ct < CT; ++ct) oacc[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[ct], pb[st], oacc[ct], 0, 0, 0);
                    __builtin_amdgcn_s_setprio(0);
                }
            }
        }
        wave_lds_sync();  // the tiles are consumed before the next iteration overwrites them
    }

    if (SPLIT) {
        // Waves 1-3 leave their state (running reference, partial sum, accumulators) in their own tile
        // buffers, lane-contiguous; wave 0 folds them into its own: with m = max of the references, every
        // state is rescaled by 2^(m_w - m) before it is added (the usual merge of online-softmax states).
        constexpr int HALF = (CT / 2) * 16 * 64;  // floats of the first CT/2 accumulators = the key tile's size
        float *sk = (float *)kt_s[wave], *sv = (float *)vt_s[wave];
        if (wave != 0) {
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float *dst = ct < CT / 2 ? sk + (ct * 16 + r) * 64 : sv + ((ct - CT / 2) * 16 + r) * 64;
                    dst[lane] = oacc[ct][r];
                }
            sv[HALF + lane] = m_run;
            sv[HALF + 64 + lane] = l_run;
        }
        __syncthreads();
        if (wave != 0) return;
#pragma unroll
        for (int w = 1; w < 4; ++w) {
            const float *ok = (const float *)kt_s[w], *ov = (const float *)vt_s[w];
            const float m_w = ov[HALF + lane], l_w = ov[HALF + 64 + lane];
            const float m_new = fmaxf(m_run, m_w);
            const float m_safe = m_new == -INFINITY ? 0.f : m_new;
            const float a = __builtin_amdgcn_exp2f(m_run - m_safe), bw = __builtin_amdgcn_exp2f(m_w - m_safe);
            l_run = l_run * a + l_w * bw;
            m_run = m_new;
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float *src = ct < CT / 2 ? ok + (ct * 16 + r) * 64 : ov + ((ct - CT / 2) * 16 + r) * 64;
                    oacc[ct][r] = oacc[ct][r] * a + src[lane] * bw;
                }
        }
    }

    // ---- normalise, transpose through LDS, coalesced store
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            uint2 u;
            u.x = pack_bf16(oacc[ct][4 * g + 0] * inv, oacc[ct][4 * g + 1] * inv);
            u.y = pack_bf16(oacc[ct][4 * g + 2] * inv, oacc[ct][4 * g + 3] * inv);
            *(uint2 *)(vt + col * PITCH + ct * 32 + g * 8 + hh * 4) = u;
        }
    wave_lds_sync();
    bf16_t *Ob = (bf16_t *)p.O + (int64_t)b * p.os_b + (int64_t)h * p.os_h + (int64_t)row0 * p.os_r;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int row = lane / CPR + i * RPI;
        if (row < n_rows) *(uint4 *)(Ob + (int64_t)row * p.os_r + (lane % CPR) * 8) = *(const uint4 *)(vt + row * PITCH + (lane % CPR) * 8);
    }
}

bool attn_mfma_supported(const KParams &p, bool bf16)
{
    // contiguous variant: a row's offset inside its (sequence, kv head) slice is kept in 32 bits of 16-byte units
    const bool fits = p.page_table || (int64_t)p.max_kv_len * p.ks_r < (1LL << 35);
    return bf16 && p.q_len > 1 && p.bk <= 16 && (p.bk & (p.bk - 1)) == 0 && p.bq <= 64 && fits;
}

hipError_t launch_attn_mfma(const KParams &p, hipStream_t st)
{
    int log_bk = 0;
    while ((1 << log_bk) < p.bk) ++log_bk;
    const int mtn = (p.bq + 31) / 32;
    const int64_t groups = (int64_t)p.batch * p.hkv;
    const int64_t per_group = (int64_t)p.g * p.nqb * mtn;
    const int64_t waves = groups * per_group;
    if (waves == 0) return hipSuccess;
    // few work items (a quarter of the GPU's wave slots or less): a workgroup per work item, four waves share its key tiles
    const bool split = waves <= 512;
    // groups worked on at a time (measured: all eight up to 128k tokens at head dim 128, four at 256k, one at a million)
    const int xcd_map = (groups % 8 == 0 && (split || per_group % 4 == 0)) ? groups_at_a_time((int64_t)p.max_kv_len * p.d * 4, 768LL << 20) : 0;
    dim3 grid((unsigned)placed_workgroups(xcd_map, split ? 1 : 4, per_group, groups)), block(kThreads);
    const int mode = p.page_table ? 1 : ((int64_t)p.max_kv_len * p.ks_r * 2 < (1LL << 32) ? 0 : 2);
#define HIPATTN_LAUNCH(DV, SP)                                                                                  \
    do {                                                                                                        \
        if (mode == 1) hipLaunchKernelGGL((attn_mfma_kernel<DV, 1, SP>), grid, block, 0, st, p, log_bk, mtn, xcd_map);      \
        else if (mode == 0) hipLaunchKernelGGL((attn_mfma_kernel<DV, 0, SP>), grid, block, 0, st, p, log_bk, mtn, xcd_map); \
        else hipLaunchKernelGGL((attn_mfma_kernel<DV, 2, SP>), grid, block, 0, st, p, log_bk, mtn, xcd_map);                \
    } while (0)
    if (p.d == 128 && p.kb <= 1024) {
        // head dim 128: the variant that loads the gathered rows straight into LDS (attn_mfma_direct.hip)
        return launch_attn_mfma_direct(p, grid, log_bk, mtn, xcd_map, mode, split, st);
    }
    if (p.d == 64) {
        if (split) HIPATTN_LAUNCH(64, true); else HIPATTN_LAUNCH(64, false);
    } else {
        if (split) HIPATTN_LAUNCH(128, true); else HIPATTN_LAUNCH(128, false);
    }
#undef HIPATTN_LAUNCH
    return hipGetLastError();
}

}  // namespace hipattn
