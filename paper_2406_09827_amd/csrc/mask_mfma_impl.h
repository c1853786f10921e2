// Hierarchical mask estimation for bf16 prefill on CDNA4 matrix cores
// (paper Alg. 1; the block approximation of Sec. 3.2 is what makes the branch scoring a
// dense query-block x gathered-key-rows contraction).
//
// Work item = one WAVE = one (sequence, query head, query block); four independent work
// items per workgroup, no workgroup barrier and no work done twice.
//   * The query block (<= 64 rows) sits in registers as the MFMA A operand.
//   * A round scores 2*kb branches = 2*kb*bk gathered key rows in tiles of 32 rows.  The rows
//     are loaded COALESCED (a row = D/8 consecutive lanes x 16 bytes, so the address unit sees
//     whole cache lines instead of 64 separate ones), parked in two alternating register sets
//     while in flight (two tiles ahead), written into the wave's LDS tile with an XOR swizzle
//     and read back in the MFMA B-operand layout (lane l: row l % 32, 16-byte chunk l / 32 of
//     each 32-byte step) without bank conflicts.  A loading lane finds the rows it loads with
//     ONE read of the branch table (its rows belong to consecutive branch slots), issued a
//     further tile ahead, so no LDS round trip sits between two tiles.  Rows of empty
//     branches load row 0 of the sequence (always mapped) and drop the result: loads stay
//     unconditional.  For one query tile, up to 1024 branch slots and keys that stay in the caches
//     (the common prefill shapes) a second form of the loop loads the rows straight into LDS
//     (global_load_lds_dwordx4): no staging registers, three waves per SIMD instead of two.
//   * Sampling strides b_sq / b_sk (powers of two) shrink the operand tiles: only the sampled query
//     rows are loaded into the A operand, only the sampled key rows of a block are gathered.
//   * v_mfma_f32_32x32x16_bf16 gives a 32(query) x 32(key) score tile; the branch score is
//     the max over the admissible query rows (in-lane, then lanes l and l+32) and over the
//     bk keys of the block (neighbouring lanes, DPP).
//   * Scores go to the wave's LDS slice as order-preserving integer keys; the wave runs the
//     ordered threshold selection, compacts the surviving nodes in place and writes, per
//     surviving node, the representative blocks of its two branches into a branch table, so
//     the scoring loop of the next round does one table lookup per key row.
// Node ranges are block indices [s, e); the list stays sorted by position throughout, which
// is why the result needs no sort.
#pragma once
#include "common.h"
#include "launch.h"

namespace hipattn {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

// max over lanes l and l ^ 32 (both get it)
__device__ __forceinline__ float max_half_swap(float v)
{
    const unsigned u = __float_as_uint(v);
    auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// MT = 32-row query tiles (1 or 2), E = branch slots / 64, D = head dim,
// LB = log2(key rows scored per block) = log2(bk / b_sk)
// SPLIT: the workgroup takes ONE work item; its four waves share the node state, score a quarter of the tiles
// each and run the selection redundantly (for launches with too few work items to fill the GPU wave by wave)
// DIRECT: the key rows go from memory straight into LDS (global_load_lds_dwordx4) instead of through registers and
// ds_write; see the tile loop.  One query tile, 512 branch slots, contiguous K only.
// SHARE4 (with DIRECT): the four waves of a workgroup are four query heads of ONE (sequence, kv head, query block).  In
// the first round they all score the same representative blocks (the initial nodes depend on the lengths only), so they
// go through that round in step: each tile is loaded once, by one of the four waves, and read by all of them.
template <int MT, int E, int D, bool PAGED, int LB, bool SPLIT = false, bool DIRECT = false, bool SHARE4 = false>
__device__ __forceinline__ void mask_mfma_body(const KParams &p, int xcd_map)
{
    static_assert(!SHARE4 || (DIRECT && !PAGED && !SPLIT), "shared first round: direct-to-LDS variant over contiguous keys");
    static_assert(!DIRECT || (MT == 1 && E <= 16 && !SPLIT && (!PAGED || E == 8)), "the direct-to-LDS variant: one query tile, up to 1024 slots (512 over a paged pool)");
    constexpr int NB = 64 * E;     // branch slots
    constexpr int KS = D / 16;     // MFMA k-steps per key row
    constexpr int BK = 1 << LB;    // key rows scored per representative block
    constexpr int CPR = D / 8;     // 16-byte chunks per key row
    constexpr int RPI = 64 / CPR;  // rows per wave-wide load
    constexpr int NLD = 32 / RPI;  // rows (= loads) per lane and tile
    constexpr int SPL = NLD >> LB; // branch slots a loading lane's rows belong to (>= 1)
    constexpr int ROWB = D * 2;    // bytes per row
    typedef uint32_t stage_t __attribute__((ext_vector_type(4 * NLD)));
    static_assert(SPL >= 1, "bk too large for this kernel");
    constexpr int NC = SPLIT ? 1 : 4;  // copies of the per-work-item state
    __shared__ uint32_t keys_s[NC][NB];
    __shared__ __attribute__((aligned(16))) int brt_s[NC][NB];        // per branch slot: first key of its centre block, -1 = empty
    // List rounds: slot of the i-th block still to be scored.  With 1024 branch slots and one query tile the
    // slot is packed into the list entry instead (slot << 21 | block index; the launcher checks that block
    // indices fit 21 bits): without this array the workgroup's LDS is 80 KB and two workgroups share a
    // compute unit.
    constexpr bool PACK = (E == 16 || DIRECT) && MT == 1;
    // With a page table: the page of every branch slot's block, looked up when the branch table is written
    // (once per round) so that the tile loop has no dependent look-up.  With 2048 slots the table does not
    // fit; the look-up is then issued from the tile loop, a few tiles ahead of the row loads.
    constexpr bool PGL = PAGED && E <= 16 && !DIRECT;
    // DIRECT over a paged pool: the sequence's row of the page table (at most 1024 pages) is copied into LDS once per
    // workgroup - the launcher sees to it that the four work items of a workgroup belong to one sequence - and the
    // tile loop looks pages up there: 4 KB instead of the 8 KB of per-slot page ids, which keeps three workgroups
    // on a compute unit.
    constexpr bool PTC = PAGED && DIRECT;
    constexpr int kMaxCachedPages = 1024;
    // one 32-row tile per wave.  DIRECT: the node ranges [s, e) share it (they are only touched between two rounds'
    // tile loops and sit in registers meanwhile); the workgroup's LDS is then 48 KB and three workgroups fit a
    // compute unit.
    constexpr int TILEB = 32 * D * 2;
    __shared__ __attribute__((aligned(16))) uint4 tile_buf[4][TILEB / 16];
    // (the LDS address of a direct load travels in M0: all of this variant's LDS stays below 64 KB)
    static_assert(!DIRECT || 2 * NC * NB * 4 + 4 * TILEB + (PTC ? 4 * kMaxCachedPages : 0) <= 65536, "LDS of the direct-to-LDS variant");

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, hh = lane >> 5;
    const int own = SPLIT ? 0 : wave;  // which copy of the state

    // ---- which (sequence, head, query block) this wave owns.  With `xcd_map` the workgroups an
    // XCD receives (blockIdx.x % 8) all read the same KV head; query blocks go from the longest
    // prefix down, the query heads of a KV group are adjacent.
    const uint32_t groups = (uint32_t)p.batch * (uint32_t)p.hkv;
    const uint32_t per_group = (uint32_t)p.g * (uint32_t)p.nqb;
    uint32_t group, o;
    if (!place_item(xcd_map, blockIdx.x, SPLIT ? 1 : 4, SPLIT ? 0 : wave, per_group, groups, group, o)) return;
    const uint32_t oq = o / (uint32_t)p.g;
    const int qb = p.nqb - 1 - (int)oq;
    const int b = (int)(group / (uint32_t)p.hkv), hk = (int)(group - (uint32_t)b * (uint32_t)p.hkv);
    const int h = hk * p.g + (int)(o - oq * (uint32_t)p.g);
    const int kb = p.kb;
    // sampling strides of the block score are powers of two here: key row n of a block is its key
    // n << ks (ks = log2 b_sk), query row i of the operand is row i << qs of the block (qs = log2 b_sq)
    const int ks = __builtin_ctz(p.b_sk), qs = __builtin_ctz(p.b_sq);
    const int lbk = LB + ks;  // log2(bk)

    const int kv_len = p.kv_lens ? p.kv_lens[b] : p.max_kv_len;
    const int row0 = qb * p.bq;
    const int n_rows = min(p.bq, p.q_len - row0);
    const int n_eff = (n_rows + p.b_sq - 1) >> qs;  // sampled query rows
    const int pos0 = kv_len - p.q_len + row0;
    const int L = min(kv_len, pos0 + n_rows);
    int32_t *out = p.idx_out + (((int64_t)b * p.hq + h) * p.nqb + qb) * kb;

    const int Tb = L > 0 ? (L + p.bk - 1) >> lbk : 0;
    if (Tb <= kb) {
        for (int j = lane; j < kb; j += 64) out[j] = j < Tb ? j << lbk : kSentinel;
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
                // operand rows past the sampled rows of the block repeat the last one: a repeated row cannot
                // change a maximum, so tiles that need no causal masking take the short reduction whatever
                // the number of rows
                const uint4 v = *(const uint4 *)(Qb + (int64_t)(min(i, n_eff - 1) << qs) * p.qs_r + kk * 16 + hh * 8);
                qf[mt][kk] = __builtin_bit_cast(bf16x8, v);
            }
        }
    }

    uint32_t *keys = keys_s[own];
    int *ns, *ne, *brt = brt_s[own], *fsl = nullptr, *bpg = nullptr;
    if constexpr (DIRECT) {
        ns = (int *)tile_buf[wave];
        ne = ns + NB / 2;
    } else {
        __shared__ int nds[NC][NB / 2], nde[NC][NB / 2];  // node ranges [s, e) in key blocks
        ns = nds[own];
        ne = nde[own];
    }
    if constexpr (!PACK) {
        __shared__ int fsl_s[NC][NB / 2];
        fsl = fsl_s[own];
    }
    if constexpr (PGL) {
        __shared__ __attribute__((aligned(16))) int bpg_s[NC][NB];
        bpg = bpg_s[own];
    }
    // (page sizes are powers of two here: no branch or division in the tile loop)
    const int *ptab = PAGED ? p.page_table + (int64_t)b * p.max_pages : nullptr;
    const int pg0 = PGL ? ptab[0] : 0;  // empty entries load key 0
    int *ptc = nullptr;
    if constexpr (PTC) {
        // every wave of the workgroup writes the same values: no workgroup barrier (waves may have left already)
        __shared__ int ptab_s[kMaxCachedPages];
        ptc = ptab_s;
        for (int i = lane; i < p.max_pages; i += 64) ptc[i] = ptab[i];
    }
    // branch-table entry i: first key `t0` of the block to score (-1: none); `word` is what the table holds
    auto set_branch = [&](int i, int word, int t0) __attribute__((always_inline)) {
        brt[i] = word;
        if (PGL) bpg[i] = t0 >= 0 ? ptab[t0 >> p.page_shift] : pg0;
        if (PAGED && p.touched && t0 >= 0) touch_page(p, b, t0);
    };
    // the waves of a work item meet here (SPLIT); otherwise the point only orders one wave's LDS traffic
    auto sync_unit = [&]() __attribute__((always_inline)) {
        if (SPLIT) __syncthreads(); else wave_lds_sync();
    };
    char *tile_s = (char *)tile_buf[wave];

    // the two branches of node [s, e): left [s, mid) (empty for a one-block node), right [mid, e);
    // each is represented by its centre block.  Written once per surviving node, so the
    // scoring loop only looks the representative up.
    auto put_branches = [&](int j, int s, int e) __attribute__((always_inline)) {
        const int mid = s + ((e - s) >> 1);
        const int l = mid > s ? rep_block(s, mid, p.rep_pos) << lbk : -1, r = rep_block(mid, e, p.rep_pos) << lbk;
        set_branch(2 * j, l, l);
        set_branch(2 * j + 1, r, r);
    };
    for (int i = lane; i < NB; i += 64) { keys[i] = 0; set_branch(i, -1, -1); }
    sync_unit();
    {
        const int a = Tb / kb, r = Tb % kb;
        for (int j = lane; j < kb; j += 64) {
            const int s = chunk_bound(j, a, r, kb), e = chunk_bound(j + 1, a, r, kb);
            ns[j] = s; ne[j] = e;
            put_branches(j, s, e);
        }
    }
    sync_unit();

    int n_tiles = (2 * kb * BK + 31) >> 5;   // every slot a tile touches is < NB
    // Rounds that run from a compact list.  A child that has its parent's representative block has the
    // parent's score, which is carried over from the round that kept the parent, and only the other
    // child is gathered and scored: with the first (last) block as representative that is the left
    // (right) child in every round after the first; with the centre representative it happens in the
    // final round, where every node is one or two blocks long, a one-block node IS its representative
    // and the right half of a two-block node is the node's representative.  In such a round the branch
    // table is a compact list of the blocks to score and fsl[] names the slot each one belongs to.
    bool final_mode = false;
    const int lg = lane / CPR, lc = lane % CPR;  // loading role: rows lg*NLD .. +NLD-1, chunk lc
    // row 0 of this sequence / kv head (contiguous layout only)
    // The slice address is the same in every lane; saying so (readfirstlane) lets the loads take it as a
    // scalar base plus a 32-bit lane offset, which is one 24-bit multiply-add per row instead of
    // 64-bit vector arithmetic (the launcher checks that rows and row pitch fit 24 bits).
    const int64_t slice = ((int64_t)b * p.ks_b + (int64_t)hk * p.ks_h) * 2;  // bytes
    const int64_t slice_u = ((int64_t)__builtin_amdgcn_readfirstlane((int)(slice >> 32)) << 32) |
                            (uint32_t)__builtin_amdgcn_readfirstlane((int)slice);
    const char *Kseq = (const char *)p.K + slice_u;
    const uint32_t row_bytes = (uint32_t)p.ks_r * 2u, lc_bytes = (uint32_t)lc * 16u;
    // paged layout: this kv head's rows of page 0, and the pitch of a page
    const int64_t head_off = (int64_t)hk * p.ks_h * 2;
    const char *Kpool = (const char *)p.K + (((int64_t)__builtin_amdgcn_readfirstlane((int)(head_off >> 32)) << 32) |
                                             (uint32_t)__builtin_amdgcn_readfirstlane((int)head_off));
    const char *Kpool_back = (const char *)p.Kback + (Kpool - (const char *)p.K);
    const uint32_t page_bytes = (uint32_t)p.ks_b * 2u;

    // Branch-table entries one tile needs: m[0..SPL-1] for the rows this lane LOADS, m[SPL] for
    // the row it SCORES (row col of the tile).
    // With a page table, pg[] holds the pages of the blocks this lane loads.
    struct meta_t { int m[SPL + 1]; int sl; int pg[PAGED ? SPL : 1]; };
    auto read_meta = [&](int tile, meta_t &mt_) __attribute__((always_inline)) {
        const int *src = brt + tile * (32 >> LB) + lg * SPL;
        if (SPL == 1) mt_.m[0] = src[0];
        else if (SPL == 2) { const int2 v = *(const int2 *)src; mt_.m[0] = v.x; mt_.m[1] = v.y; }
        else {
#pragma unroll
            for (int i = 0; i < SPL; i += 4) {
                const int4 v = *(const int4 *)(src + i);
                mt_.m[i] = v.x; mt_.m[i + 1] = v.y; mt_.m[i + 2] = v.z; mt_.m[i + 3] = v.w;
            }
        }
        mt_.m[SPL] = brt[(tile * 32 + col) >> LB];
        const int ti = (tile * 32 + col) >> LB;
        if (PACK) {
            mt_.sl = final_mode ? mt_.m[SPL] >> 21 : ti;
            if (final_mode) {
#pragma unroll
                for (int i = 0; i <= SPL; ++i) mt_.m[i] = mt_.m[i] < 0 ? -1 : (mt_.m[i] & 0x1fffff) << lbk;
            }
        } else {
            mt_.sl = final_mode ? fsl[min(ti, NB / 2 - 1)] : ti;  // (entries past the list are never used)
        }
        if (PGL) {
            const int *pgs = bpg + tile * (32 >> LB) + lg * SPL;
            if (SPL == 1) mt_.pg[0] = pgs[0];
            else if (SPL == 2) { const int2 v = *(const int2 *)pgs; mt_.pg[0] = v.x; mt_.pg[1] = v.y; }
            else {
#pragma unroll
                for (int i = 0; i < SPL; i += 4) {
                    const int4 v = *(const int4 *)(pgs + i);
                    mt_.pg[i] = v.x; mt_.pg[i + 1] = v.y; mt_.pg[i + 2] = v.z; mt_.pg[i + 3] = v.w;
                }
            }
        } else if (PTC) {
#pragma unroll
            for (int i = 0; i < SPL; ++i) mt_.pg[i] = ptc[max(mt_.m[i], 0) >> p.page_shift];
        } else if (PAGED) {
#pragma unroll
            for (int i = 0; i < SPL; ++i) mt_.pg[i] = ptab[max(mt_.m[i], 0) >> p.page_shift];
        }
    };

    // Row info of a tile from the metadata read earlier: t = key position of this lane's scored row,
    // or -1 if the row does not count; slot = its branch slot, complemented when the branch is empty.
    auto row_info = [&](const meta_t &mt_, int &t, int &slot) __attribute__((always_inline)) {
        const int sl = mt_.sl, tf = mt_.m[SPL];
        const int tt = tf + ((col & (BK - 1)) << ks);
        t = (tf >= 0 && tt < kv_len) ? tt : -1;
        // empty: in a normal round the slot is still named (complemented) so its key gets cleared;
        // in the final round an entry past the end of the list names no slot at all
        slot = tf >= 0 ? sl : (final_mode ? -1 : ~sl);
    };
    // Coalesced load of row j (of NLD) of this lane's share of a tile.  Rows past the end of the
    // sequence re-read its last row (their score is dropped: t < 0 in row_info).
    auto load_row = [&](const meta_t &mt_, stage_t &R, int j) __attribute__((always_inline)) {
        const int i = j / BK, n = j % BK;
        const int tf = max(mt_.m[i], 0);
        const int last = kv_len - 1;
        uint4 x;
        if (PAGED) {
            // a block never straddles a page
            // a block never straddles a page: page base (one 64-bit multiply-add per block) plus a
            // 32-bit offset inside the page
            const int in_page = tf & (p.page_size - 1);
            const uint32_t r = (uint32_t)(in_page + min(tf + (n << ks), last) - tf);
            // (a negative page-table entry names a page of the backing pool)
            const char *pb = (mt_.pg[i] < 0 ? Kpool_back : Kpool) + (uint64_t)(uint32_t)page_in_pool(mt_.pg[i]) * page_bytes;
            x = *(const uint4 *)(pb + (__umul24(r, row_bytes) + lc_bytes));
        } else {
            x = *(const uint4 *)(Kseq + (__umul24((uint32_t)min(tf + (n << ks), last), row_bytes) + lc_bytes));
        }
        R[4 * j] = x.x; R[4 * j + 1] = x.y; R[4 * j + 2] = x.z; R[4 * j + 3] = x.w;
    };
    auto load_rows = [&](const meta_t &mt_, stage_t &R, int &t, int &slot) __attribute__((always_inline)) {
        row_info(mt_, t, slot);
#pragma unroll
        for (int j = 0; j < NLD; ++j) load_row(mt_, R, j);
    };

    // registers -> swizzled LDS tile: row r = lg*NLD + j, chunk lc goes to slot lc ^ (r % CPR)
    auto park_row = [&](const stage_t &R, int j) __attribute__((always_inline)) {
        const int r = lg * NLD + j;
        *(uint4 *)(tile_s + r * ROWB + ((lc ^ (r & (CPR - 1))) << 4)) =
            make_uint4(R[4 * j], R[4 * j + 1], R[4 * j + 2], R[4 * j + 3]);
    };
    auto park = [&](const stage_t &R) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < NLD; ++j) park_row(R, j);
    };

    struct acc_t { f32x16 a[MT]; };
    // Branch score from a tile of products, written as an ordered key
    auto score_finish = [&](const acc_t &A, int t, int slot) __attribute__((always_inline)) {
        const f32x16 (&acc)[MT] = A.a;
        // max over the admissible query rows of this lane's key column
        const int lo = t - pos0;  // block rows below lo would look into the future
        float v = -INFINITY;
        if (__ballot(lo > 0) == 0) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                float w[4];
#pragma unroll
                for (int g = 0; g < 4; ++g) w[g] = fmaxf(fmaxf(acc[mt][4 * g], acc[mt][4 * g + 1]), fmaxf(acc[mt][4 * g + 2], acc[mt][4 * g + 3]));
                v = fmaxf(v, fmaxf(fmaxf(w[0], w[1]), fmaxf(w[2], w[3])));
            }
        } else {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int i = mt * 32 + (r >> 2) * 8 + hh * 4 + (r & 3);
                    if ((i << qs) >= lo && i < n_eff) v = fmaxf(v, acc[mt][r]);
                }
        }
        if (t < 0) v = -INFINITY;
        v = max_half_swap(v);
        if (LB >= 1) v = fmaxf(v, dpp_f<0xB1>(v));  // lane ^ 1
        if (LB >= 2) v = fmaxf(v, dpp_f<0x4E>(v));  // lane ^ 2
        if (LB >= 3) v = fmaxf(v, dpp_f<0x141>(v)); // lane i <-> 7 - i of each 8 lanes: the other quad (quads are uniform by now)
        const int sl = slot < 0 ? ~slot : slot;
        // (in the final round the keys are preset and an empty entry names no slot)
        if (hh == 0 && (col & (BK - 1)) == 0 && (slot >= 0 || !final_mode)) keys[sl] = slot < 0 ? 0u : score_key(v);
    };

    static_assert(NLD == KS, "one staged row per k-step");
    // One pipeline step: multiplies the tile that sits in LDS (operands are read into registers first)
    // and, between the multiplies, moves the staged tile R into the LDS tile row by row and refills R
    // with the rows of the tile named by mt_.  The order is pinned: left to itself the compiler issues
    // the multiplies back to back, and the wave then waits on the matrix pipe with all of this
    // independent work behind it.
    auto multiply_and_restage = [&](acc_t &A, stage_t &R, const meta_t &mt_, int &t, int &slot) __attribute__((always_inline)) {
        f32x16 (&acc)[MT] = A.a;
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        // all operand reads first (one LDS latency per tile, not one per k-step)
        uint4 kv[KS];
#pragma unroll
        for (int kk = 0; kk < KS; ++kk)
            kv[kk] = *(const uint4 *)(tile_s + col * ROWB + (((kk * 2 + hh) ^ (col & (CPR - 1))) << 4));
        row_info(mt_, t, slot);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[mt][kk], __builtin_bit_cast(bf16x8, kv[kk]), kk == 0 ? zero : acc[mt], 0, 0, 0);
            park_row(R, kk);
            load_row(mt_, R, kk);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    if constexpr (DIRECT) {
        // The query loads end here, where the compiler can see it: it does not count the loads that the tile loop
        // issues from inline assembly, and a wait for a query fragment left inside that loop would wait for them.
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) asm volatile("" :: "v"(qf[0][kk]));
    }
    // ensemble sample: the round whose selection compares perturbed scores (-1: none)
    const int ens_round = ens_round_of(p.ens_sample, (Tb + kb - 1) / kb);
    const uint32_t ens_hash = ens_round >= 0 ? ens_unit_hash(p.ens_seed, p.ens_sample, b, h, qb) : 0u;
    int round = 0;
    for (int maxlen = (Tb + kb - 1) / kb; maxlen > 1; maxlen = (maxlen + 1) >> 1, ++round) {
        // Pipeline: branch-table reads run three to four tiles ahead of the multiply, row loads two.
        // The loop body is straight-line code: tile numbers past the end are clamped to the last tile
        // (it is then loaded and scored again, which rewrites the same keys), because a load that is
        // issued on some paths only makes the compiler wait for ALL outstanding loads before it
        // touches a staged register, and that exposes the full memory latency in every tile.
        // With SPLIT, wave w takes tiles w, w + 4, ...: tile_of(i) is the i-th tile of this wave.
        const int nt_all = __builtin_amdgcn_readfirstlane(n_tiles);
        const int nt = SPLIT ? (nt_all > wave ? (nt_all - wave + 3) >> 2 : 0) : nt_all;
        if constexpr (DIRECT) {
            // Direct-to-LDS variant: a global load that delivers into LDS (lane l's 16 bytes land at M0 + 16 l)
            // needs neither staging registers nor a ds_write, so this variant runs in 160 registers and 48 KB of
            // LDS (head dim 128): three waves per SIMD instead of two.  Load j of a tile fills 1 KB of LDS, i.e. LDS
            // rows RPI j .. RPI j + RPI - 1 (RPI = 4 rows of 256 bytes, or 8 of 128); lane group lg supplies tile
            // row lg * NLD + j (the rows a lane loads belong to consecutive branch slots, as in the other variant),
            // so tile row r sits in LDS row RPI (r % NLD) + r / NLD, and the XOR swizzle is applied to the global
            // chunk a lane fetches.  The wave has one tile buffer: as soon as a tile's operands are in registers the
            // buffer is refilled with the next tile, which lands while this one is multiplied and scored.  The loads
            // are inline assembly with explicit waits: the compiler neither sees that they write LDS nor counts
            // them, and no other vector memory instruction is issued inside the loop.
            int sv[E];  // node ranges, out of the way of the tiles
#pragma unroll
            for (int i = 0; i < E / 2; ++i) { sv[i] = ns[i * 64 + lane]; sv[E / 2 + i] = ne[i * 64 + lane]; }
            asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
            if (nt > 0) {
                const int last_tile = nt - 1;
                auto tile_of = [&](int i) __attribute__((always_inline)) { return min(i, last_tile); };
                const uint32_t ring = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)tile_buf[wave];
                const int last = kv_len - 1;
                // one load: row j of this lane's share of the tile described by mt_, into buffer `buf`.  (M0 is a
                // reserved register: the compiler warns that it does not track the clobber.  It is written and
                // consumed inside one asm statement, and nothing else in these kernels uses M0.)
                auto issue_row = [&](const meta_t &mt_, int buf, int j) __attribute__((always_inline)) {
                    const int i = j / BK, n = j % BK;
                    const int tf = max(mt_.m[i], 0);
                    const int rho = lg * NLD + j;
                    const uint32_t chunk = (uint32_t)((lc ^ (rho & (CPR - 1))) << 4);
                    const uint32_t dst = __builtin_amdgcn_readfirstlane(ring + buf * TILEB + j * 1024);
                    if constexpr (PAGED) {
                        // page base (the resident pool, or the backing pool for a negative entry) plus a 32-bit offset inside the page
                        const uint32_t r = (uint32_t)((tf & (p.page_size - 1)) + min(tf + (n << ks), last) - tf);
                        const char *src = (mt_.pg[i] < 0 ? Kpool_back : Kpool) + (uint64_t)(uint32_t)page_in_pool(mt_.pg[i]) * page_bytes +
                                          (__umul24(r, row_bytes) + chunk);
                        asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                                     :: "v"(src), "s"(dst) : "memory", "m0");
                    } else {
                        const uint32_t voff = __umul24((uint32_t)min(tf + (n << ks), last), row_bytes) + chunk;
                        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                                     :: "v"(voff), "s"(Kseq), "s"(dst) : "memory", "m0");
                    }
                };
                // operands of the tile in buffer `buf`: tile row `col` sits in LDS row RPI (col % NLD) + col / NLD
                auto read_operands = [&](int buf, uint4 (&kv)[KS]) __attribute__((always_inline)) {
                    const uint32_t base = ring + buf * TILEB + (RPI * (col % NLD) + col / NLD) * ROWB;
#pragma unroll
                    for (int kk = 0; kk < KS; ++kk)
                        asm volatile("ds_read_b128 %0, %1" : "=v"(kv[kk]) : "v"(base + (((kk * 2 + hh) ^ (col & (CPR - 1))) << 4)) : "memory");
                };
                // One step: the tile in the buffer is multiplied and, as soon as its operands are in registers,
                // the buffer is refilled with the next tile (described by mt_, whose row info comes back in t / slot).
                auto step = [&](acc_t &A, meta_t &mt_, int &t, int &slot, int next_meta_tile) __attribute__((always_inline)) {
                    f32x16 (&acc)[MT] = A.a;
                    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the tile has landed
                    uint4 kv[KS];
                    read_operands(0, kv);
                    row_info(mt_, t, slot);
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // operands are in registers: the buffer may be refilled
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int kk = 0; kk < KS; ++kk) {
                        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[0][kk], __builtin_bit_cast(bf16x8, kv[kk]), kk == 0 ? zero : acc[0], 0, 0, 0);
                        issue_row(mt_, 0, kk);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    read_meta(next_meta_tile, mt_);
                };
                if (SHARE4 && round == 0) {
                    // First round, shared: tile t is loaded by wave t % 4 into ITS buffer (three steps ahead) and read
                    // by all four waves.  One barrier per step: it says that tile t has landed (its owner waited for
                    // it) and that every wave has the operands of tile t-1 in registers, so that buffer may be refilled.
                    const uint32_t ring0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)tile_buf[0];
                    meta_t ml;
                    if (wave < nt) {
                        read_meta(wave, ml);
#pragma unroll
                        for (int j = 0; j < NLD; ++j) issue_row(ml, 0, j);
                    }
                    for (int t = 0; t < nt; ++t) {
                        const int ow = t & 3;
                        if (wave == ow) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                        __builtin_amdgcn_s_barrier();
                        uint4 kv[KS];
                        {
                            const uint32_t base = ring0 + ow * TILEB + (RPI * (col % NLD) + col / NLD) * ROWB;
#pragma unroll
                            for (int kk = 0; kk < KS; ++kk)
                                asm volatile("ds_read_b128 %0, %1" : "=v"(kv[kk]) : "v"(base + (((kk * 2 + hh) ^ (col & (CPR - 1))) << 4)) : "memory");
                        }
                        meta_t ms;
                        int tcur, scur;
                        read_meta(t, ms);
                        row_info(ms, tcur, scur);
                        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                        __builtin_amdgcn_sched_barrier(0);
                        if (t >= 1 && wave == ((t - 1) & 3) && t + 3 < nt) {
                            read_meta(t + 3, ml);
#pragma unroll
                            for (int j = 0; j < NLD; ++j) issue_row(ml, 0, j);
                        }
                        acc_t A;
                        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int kk = 0; kk < KS; ++kk)
                            A.a[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[0][kk], __builtin_bit_cast(bf16x8, kv[kk]), kk == 0 ? zero : A.a[0], 0, 0, 0);
                        score_finish(A, tcur, scur);
                    }
                    // the node ranges go back into the tile buffers next: not before every wave has read its last tiles
                    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
                    __builtin_amdgcn_s_barrier();
                } else {
                meta_t m0, m1;
                int tc, sc, tn, sn;
                read_meta(tile_of(0), m0);
                read_meta(tile_of(1), m1);
                row_info(m0, tc, sc);
#pragma unroll
                for (int j = 0; j < NLD; ++j) issue_row(m0, 0, j);
                read_meta(tile_of(2), m0);
                for (int tile = 0; tile < nt; tile += 2) {
                    // here: the buffer holds (or is receiving) tile `tile` (row info tc/sc); m1 and m0 hold the
                    // branch-table entries of tile+1 and tile+2
                    acc_t A;
                    step(A, m1, tn, sn, tile_of(tile + 3));
                    score_finish(A, tc, sc);
                    acc_t B;
                    step(B, m0, tc, sc, tile_of(tile + 4));
                    score_finish(B, tn, sn);
                }
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                }
            }
#pragma unroll
            for (int i = 0; i < E / 2; ++i) { ns[i * 64 + lane] = sv[i]; ne[i * 64 + lane] = sv[E / 2 + i]; }
        } else
        if (nt > 0) {
            const int last_tile = nt - 1;
            auto tile_of = [&](int i) __attribute__((always_inline)) { return SPLIT ? wave + 4 * min(i, last_tile) : min(i, last_tile); };
            stage_t R0, R1;  // one vector value each, so the staged rows stay in registers
            meta_t m0, m1;
            int t0, s0, t1, s1;
            read_meta(tile_of(0), m0);
            read_meta(tile_of(1), m1);
            load_rows(m0, R0, t0, s0);
            read_meta(tile_of(2), m0);
            load_rows(m1, R1, t1, s1);
            read_meta(tile_of(3), m1);
            // tile 0 goes into the LDS tile; from then on the tile after the one being multiplied is
            // written to LDS (and the loads of the tile three ahead are issued) between the multiplies
            int tcur = t0, scur = s0;
            park(R0);
            load_rows(m0, R0, t0, s0);
            read_meta(tile_of(4), m0);
            wave_lds_sync();
            for (int tile = 0; tile < nt; tile += 2) {
                // here: tile `tile` is in LDS (its row info in tcur/scur), R1 holds tile+1, R0 tile+2,
                // m1 the branch-table entries of tile+3, m0 those of tile+4
                acc_t A;
                const int tn = t1, sn = s1;
                multiply_and_restage(A, R1, m1, t1, s1);
                read_meta(tile_of(tile + 5), m1);
                wave_lds_sync();
                score_finish(A, tcur, scur);
                // tile+1 is in LDS, R0 holds tile+2, R1 tile+3
                acc_t B;
                tcur = t0; scur = s0;
                multiply_and_restage(B, R0, m0, t0, s0);
                read_meta(tile_of(tile + 6), m0);
                wave_lds_sync();
                score_finish(B, tn, sn);
            }
        }
        sync_unit();  // every score of the round is in place

        // ordered top-kb selection; survivors are compacted in place: every lane first reads the
        // parents of the slots it keeps, then (after all reads) writes the new nodes and their branches
        uint32_t key[E];
        bool keep[E];
        int dest[E];
#pragma unroll
        for (int i = 0; i < E; ++i) key[i] = keys[i * 64 + lane];
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
        int cs[E], ce[E];
#pragma unroll
        for (int i = 0; i < E; ++i) {
            cs[i] = 0; ce[i] = 0;
            if (keep[i]) {
                const int slot = i * 64 + lane, node = slot >> 1;
                const int s = ns[node], e = ne[node];
                const int mid = s + ((e - s) >> 1);
                cs[i] = (slot & 1) ? mid : s;
                ce[i] = (slot & 1) ? e : mid;
            }
        }
        // Next round as a compact list: always once the first or last block represents a branch (one
        // child of every node then has the node's own representative and keeps its score), and for the
        // centre representative in the final round (see above).
        const bool next_is_final = p.rep_pos != 0 || ((maxlen + 1) >> 1) == 2;
        const bool first_rule = p.rep_pos == 1;
        if (next_is_final) {
            // the branch table becomes the compact list of blocks still to be scored
            for (int i = lane; i < 2 * kb; i += 64) set_branch(i, -1, -1);
        }
        sync_unit();
        if (!next_is_final) {
#pragma unroll
            for (int i = 0; i < E; ++i) {
                if (keep[i]) {
                    ns[dest[i]] = cs[i];
                    ne[dest[i]] = ce[i];
                    put_branches(dest[i], cs[i], ce[i]);
                }
            }
        } else {
            int n_todo = 0;
#pragma unroll
            for (int i = 0; i < E; ++i) {
                const bool two = keep[i] && ce[i] - cs[i] > 1;  // both children exist
                const uint64_t b2 = __ballot(two);
                if (keep[i]) {
                    const int d = dest[i];
                    ns[d] = cs[i];
                    ne[d] = ce[i];
                    // the child that shares the node's representative keeps the node's score: the left one
                    // under the first-block rule (the node itself if it is one block long), else the right
                    // one; the other child is empty or goes on the list (its representative: the block
                    // at the split under the first-block rule, the block before the split otherwise)
                    const int mid = cs[i] + ((ce[i] - cs[i]) >> 1);
                    const int carried = (first_rule && two) ? 2 * d : 2 * d + 1;
                    keys[carried] = key[i];
                    keys[carried ^ 1] = 0u;
                    if (two) {
                        const int ti = n_todo + lane_prefix_count(b2);
                        const int blk = first_rule ? mid : mid - 1;
                        if (PACK) set_branch(ti, ((carried ^ 1) << 21) | blk, blk << lbk);
                        else { set_branch(ti, blk << lbk, blk << lbk); fsl[ti] = carried ^ 1; }
                    }
                }
                n_todo += __popcll(b2);
            }
            for (int i = 2 * kb + lane; i < NB; i += 64) keys[i] = 0u;
            final_mode = true;
            n_tiles = (n_todo * BK + 31) >> 5;
        }
        sync_unit();
    }

    for (int j = lane; j < kb; j += 64) out[j] = ns[j] << lbk;
}

// One query tile: two waves per SIMD (register budget 256); two query tiles: one wave per SIMD.
template <int E, int D, bool PAGED, int LB>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2))) void mask_mfma_kernel_q32(KParams p, int xcd_map)
{
    mask_mfma_body<1, E, D, PAGED, LB>(p, xcd_map);
}
// The same with direct-to-LDS loads (contiguous K, block indices below 2^21): three waves per SIMD with 512 branch
// slots (k/bk <= 256), two with 1024 (k/bk <= 512; the register-staged kernel runs one there)
template <int D, int LB>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(3))) void mask_mfma_kernel_q32_direct(KParams p, int xcd_map)
{
    mask_mfma_body<1, 8, D, false, LB, false, true>(p, xcd_map);
}
template <int D, int LB>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(3))) void mask_mfma_kernel_q32_direct_shared(KParams p, int xcd_map)
{
    mask_mfma_body<1, 8, D, false, LB, false, true, true>(p, xcd_map);
}
template <int D, int LB>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(3))) void mask_mfma_kernel_q32_direct_paged(KParams p, int xcd_map)
{
    mask_mfma_body<1, 8, D, true, LB, false, true>(p, xcd_map);
}
template <int D, int LB>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2))) void mask_mfma_kernel_q32_direct_1k(KParams p, int xcd_map)
{
    mask_mfma_body<1, 16, D, false, LB, false, true>(p, xcd_map);
}
template <int E, int D, bool PAGED, int LB>
__global__ __launch_bounds__(kThreads) void mask_mfma_kernel_q64(KParams p, int xcd_map)
{
    mask_mfma_body<2, E, D, PAGED, LB>(p, xcd_map);
}
// Few work items: a workgroup per work item (see SPLIT above)
template <int E, int D, bool PAGED, int LB>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2))) void mask_mfma_kernel_q32_split(KParams p, int xcd_map)
{
    mask_mfma_body<1, E, D, PAGED, LB, true>(p, xcd_map);
}
template <int E, int D, bool PAGED, int LB>
__global__ __launch_bounds__(kThreads) void mask_mfma_kernel_q64_split(KParams p, int xcd_map)
{
    mask_mfma_body<2, E, D, PAGED, LB, true>(p, xcd_map);
}
// k/bk above 512: the per-wave state alone fills the LDS of a compute unit (one wave per SIMD), and
// the selection holds 32 keys per lane, so the one-tile kernel runs without the two-wave register cap
template <int E, int D, bool PAGED, int LB>
__global__ __launch_bounds__(kThreads) void mask_mfma_kernel_q32_wide(KParams p, int xcd_map)
{
    mask_mfma_body<1, E, D, PAGED, LB>(p, xcd_map);
}

template <int MT, int D, int LB>
static hipError_t launch_mask_mfma_e(const KParams &p, int xcd_map, dim3 grid, bool split, bool one_sequence_per_workgroup, hipStream_t st)
{
    dim3 block(kThreads);
    // the page-table variant is a separate instantiation: a table read in the row-offset code
    // would otherwise put a full memory wait into the contiguous path's load pipeline
#define HIPATTN_LAUNCH(KERNEL, EV)                                                                     \
    do {                                                                                               \
        if (p.page_table) hipLaunchKernelGGL((KERNEL<EV, D, true, LB>), grid, block, 0, st, p, xcd_map);  \
        else hipLaunchKernelGGL((KERNEL<EV, D, false, LB>), grid, block, 0, st, p, xcd_map);           \
    } while (0)
    if (split) {
        if constexpr (MT == 1) {
            if (p.kb <= 256) HIPATTN_LAUNCH(mask_mfma_kernel_q32_split, 8);
            else HIPATTN_LAUNCH(mask_mfma_kernel_q32_split, 16);
        } else {
            if (p.kb <= 256) HIPATTN_LAUNCH(mask_mfma_kernel_q64_split, 8);
            else HIPATTN_LAUNCH(mask_mfma_kernel_q64_split, 16);
        }
    } else if constexpr (MT == 1) {
        // (up to 32 MB of keys per kv head, 128k tokens at head dim 128: beyond that the kernel waits on the memory
        // side and the deeper prefetch of the register-staged variant makes up for the third wave - measured
        // direct / staged at 48k 3.29 / 3.75 ms, 64k 4.81 / 5.43, 96k 9.20 / 9.58, 128k 14.72 / 15.00, 256k 41.9 / 41.8)
        const bool direct = !p.page_table && (int64_t)p.max_kv_len * p.ks_r * 2 <= (32 << 20);
        const bool direct_paged = p.page_table && p.kb <= 256 && p.max_pages <= 1024 && one_sequence_per_workgroup &&
                                  (int64_t)p.max_kv_len * p.ks_r * 2 <= (16 << 20);
        if (direct_paged) hipLaunchKernelGGL((mask_mfma_kernel_q32_direct_paged<D, LB>), grid, block, 0, st, p, xcd_map);
        // (the four work items of a workgroup are then four heads of one query block: they share the first round's tiles)
        else if (direct && p.kb <= 256 && one_sequence_per_workgroup && p.g % 4 == 0 && !(p.flags & 2))
            hipLaunchKernelGGL((mask_mfma_kernel_q32_direct_shared<D, LB>), grid, block, 0, st, p, xcd_map);
        else if (direct && p.kb <= 256) hipLaunchKernelGGL((mask_mfma_kernel_q32_direct<D, LB>), grid, block, 0, st, p, xcd_map);
        else if (direct && p.kb <= 512) hipLaunchKernelGGL((mask_mfma_kernel_q32_direct_1k<D, LB>), grid, block, 0, st, p, xcd_map);
        else if (p.kb <= 256) HIPATTN_LAUNCH(mask_mfma_kernel_q32, 8);
        else if (p.kb <= 512) HIPATTN_LAUNCH(mask_mfma_kernel_q32, 16);
        else HIPATTN_LAUNCH(mask_mfma_kernel_q32_wide, 32);
    } else {
        if (p.kb <= 256) HIPATTN_LAUNCH(mask_mfma_kernel_q64, 8);
        else if (p.kb <= 512) HIPATTN_LAUNCH(mask_mfma_kernel_q64, 16);
        else HIPATTN_LAUNCH(mask_mfma_kernel_q64, 32);
    }
#undef HIPATTN_LAUNCH
    return hipGetLastError();
}

// One translation unit per key-block size instantiates this.
template <int LB> hipError_t launch_mask_mfma_lb(const KParams &p, hipStream_t st)
{
    const int64_t groups = (int64_t)p.batch * p.hkv;
    const int64_t per_group = (int64_t)p.g * p.nqb;
    const int64_t units = groups * per_group;
    if (units == 0) return hipSuccess;
    // Few work items (a quarter of the GPU's 2048 wave slots or less): a workgroup per work item, four
    // waves sharing its tiles; measured faster up to 512 work items, level from there to 1024.
    const bool split = units <= 512 && p.kb <= 512;
    // groups worked on at a time: as many as keep the key rows in flight inside the memory-side cache
    const int xcd_map = (groups % 8 == 0 && (split || per_group % 4 == 0)) ? groups_at_a_time((int64_t)p.max_kv_len * p.d * 2, 160LL << 20) : 0;
    dim3 grid((unsigned)placed_workgroups(xcd_map, split ? 1 : 4, per_group, groups));
    const bool one_tile = (p.bq + p.b_sq - 1) / p.b_sq <= 32;
    // the four work items of a workgroup are consecutive items of one (sequence, kv head) group
    const bool one_seq = !split && per_group % 4 == 0;
    if constexpr (LB <= 2) {  // (with 64 channels a lane loads 4 rows of a tile, fewer than an 8-row block)
        if (p.d == 64) return one_tile ? launch_mask_mfma_e<1, 64, LB>(p, xcd_map, grid, split, one_seq, st) : launch_mask_mfma_e<2, 64, LB>(p, xcd_map, grid, split, one_seq, st);
    }
    return one_tile ? launch_mask_mfma_e<1, 128, LB>(p, xcd_map, grid, split, one_seq, st) : launch_mask_mfma_e<2, 128, LB>(p, xcd_map, grid, split, one_seq, st);
}

}  // namespace hipattn
