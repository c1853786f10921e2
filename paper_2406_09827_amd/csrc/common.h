// Shared device helpers of the HiP attention kernels (gfx950 only, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hipattn {

constexpr int kSentinel = 0x7fffffff;
constexpr int kThreads = 256;  // every kernel here runs 4 waves of 64 lanes per workgroup

// Kernel-side view of one call; filled by the host entry points after validation.
struct KParams {
    const void *Q, *K, *V;
    void *O;
    int32_t *idx_out;          // mask estimation output
    const int32_t *idx_in;     // sparse attention input
    const int32_t *kv_lens;    // [batch] or nullptr
    const int32_t *page_table; // [batch, max_pages] or nullptr
    const void *Kback, *Vback; // backing pools for page-table entries < 0 (entry e names page ~e), or nullptr
    uint8_t *touched;          // [batch, max_pages] or nullptr: 1 is stored for every logical page read
    int64_t qs_b, qs_h, qs_r;  // element strides
    int64_t ks_b, ks_h, ks_r;
    int64_t os_b, os_h, os_r;
    int32_t batch, hq, hkv, g, d, q_len, max_kv_len, kb, bq, bk, nqb, page_size, max_pages;
    int32_t page_shift;        // log2(page_size) when it is a power of two, else -1
    int32_t n_sink, n_window;  // sparse attention: always-attended first / most recent keys
    int32_t b_sq, b_sk;        // mask estimation: row / key sampling strides of the block score (>= 1)
    int32_t rep_pos;           // mask estimation: representative block of a branch: 0 centre, 1 first, 2 last
    int32_t top_r;             // mask estimation: channels kept per query row, 0 = all
    int32_t ens_sample;        // mask estimation: ensemble sample number, 0 = the plain mask
    uint32_t ens_seed;         // mask estimation: seed of the ensemble samples' draws
    float ens_r;               // mask estimation: size of the score perturbation of a sample > 0
    float sm_scale;
    int32_t flags;             // HIP_ATTN_* flags of the call
};

typedef uint16_t bf16_t;  // raw bfloat16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t x) { return __uint_as_float(((uint32_t)x) << 16); }

// round-to-nearest-even float -> bf16 (finite inputs)
__device__ __forceinline__ bf16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

template <typename T> __device__ __forceinline__ float ld_f32(const T *p);
template <> __device__ __forceinline__ float ld_f32<float>(const float *p) { return *p; }
template <> __device__ __forceinline__ float ld_f32<bf16_t>(const bf16_t *p) { return bf16_to_f32(*p); }

template <typename T> __device__ __forceinline__ void st_f32(T *p, float v);
template <> __device__ __forceinline__ void st_f32<float>(float *p, float v) { *p = v; }
template <> __device__ __forceinline__ void st_f32<bf16_t>(bf16_t *p, float v) { *p = f32_to_bf16(v); }

// Order-preserving map of a finite-or-infinite float onto uint32 keys > 0; key 0 is
// reserved for "empty branch".  -0 and +0 get the same key.
__device__ __forceinline__ uint32_t score_key(float f)
{
    if (f == 0.0f) f = 0.0f;
    uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Element offset of logical key/value row t of sequence b, kv head h inside its pool; `miss` says that the
// page-table entry is negative, i.e. that the row lives in the backing pool (entry e names page ~e of it).
__device__ __forceinline__ int64_t kv_row_offset(const KParams &p, int b, int h, int t, bool &miss)
{
    miss = false;
    if (p.page_table) {
        int pi, in_page;
        if (p.page_shift >= 0) { pi = t >> p.page_shift; in_page = t & (p.page_size - 1); }
        else { pi = t / p.page_size; in_page = t - pi * p.page_size; }
        const int e = p.page_table[(int64_t)b * p.max_pages + pi];
        miss = e < 0;
        return (int64_t)(e < 0 ? ~e : e) * p.ks_b + (int64_t)h * p.ks_h + (int64_t)in_page * p.ks_r;
    }
    return (int64_t)b * p.ks_b + (int64_t)h * p.ks_h + (int64_t)t * p.ks_r;
}
// Logical page of key t.
__device__ __forceinline__ int logical_page(const KParams &p, int t)
{
    return p.page_shift >= 0 ? (t >> p.page_shift) : (t / p.page_size);
}
// Marks the logical page of key t of sequence b as read (callers check p.touched first).
__device__ __forceinline__ void touch_page(const KParams &p, int b, int t)
{
    p.touched[(int64_t)b * p.max_pages + logical_page(p, t)] = 1;
}
// The pool a page-table entry points into, and the page inside it.
__device__ __forceinline__ const void *pool_of(int entry, const void *pool, const void *backing)
{
    return entry < 0 ? backing : pool;
}
__device__ __forceinline__ int page_in_pool(int entry) { return entry < 0 ? ~entry : entry; }

// The same in two steps, for kernels that want all page-table reads of a batch of rows in
// flight before the first dependent row load is issued (a dependent load in the middle of a
// batch makes the wave wait for every older load as well).
template <bool PAGED> __device__ __forceinline__ int page_of_row(const KParams &p, int b, int t)
{
    if (!PAGED) return 0;
    const int pi = p.page_shift >= 0 ? (t >> p.page_shift) : (t / p.page_size);
    return p.page_table[(int64_t)b * p.max_pages + pi];
}
template <bool PAGED> __device__ __forceinline__ int64_t row_offset_in(const KParams &p, int b, int h, int t, int page)
{
    if (!PAGED) return (int64_t)b * p.ks_b + (int64_t)h * p.ks_h + (int64_t)t * p.ks_r;
    const int in_page = p.page_shift >= 0 ? (t & (p.page_size - 1)) : (t % p.page_size);
    return (int64_t)page * p.ks_b + (int64_t)h * p.ks_h + (int64_t)in_page * p.ks_r;
}
// Element offset of row t from the start of the resident pool when the page-table entry may be negative:
// `delta` is the distance (in elements) from the resident pool to the backing pool.
template <bool PAGED> __device__ __forceinline__ int64_t row_offset_bank(const KParams &p, int b, int h, int t, int entry, int64_t delta)
{
    if (!PAGED) return row_offset_in<false>(p, b, h, t, 0);
    return row_offset_in<true>(p, b, h, t, entry < 0 ? ~entry : entry) + (entry < 0 ? delta : 0);
}

__device__ __forceinline__ int lane_prefix_count(uint64_t mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}

// Representative block of the branch [bs, be) (be > bs).
__device__ __forceinline__ int rep_block(int bs, int be, int rep_pos)
{
    return rep_pos == 1 ? bs : rep_pos == 2 ? be - 1 : bs + ((be - bs) >> 1);
}

// ---- ensemble samples (paper appendix "Ensemble Hierarchical Top-k Approximation") ------------------
// A sample e > 0 differs from the plain mask in ONE round of the search, the middle one (round R / 2 of the
// R rounds the query block runs, counted from 0): there the top-kb selection compares score + r_e * u, u a
// draw on [-1, 1) that depends only on (seed, sample, sequence, head, query block, representative block of
// the branch): MurmurHash3's 32-bit finalizer absorbs these numbers one after the other and the top 24 bits
// of the result, as an integer n, give u = (n - 2^23) / 2^23.  Product and sum are each rounded once to fp32.
__device__ __forceinline__ uint32_t fmix32(uint32_t x)
{
    x ^= x >> 16; x *= 0x85ebca6bu; x ^= x >> 13; x *= 0xc2b2ae35u; x ^= x >> 16;
    return x;
}
// everything but the representative block absorbed
__device__ __forceinline__ uint32_t ens_unit_hash(uint32_t seed, int sample, int b, int h, int qb)
{
    uint32_t x = fmix32(seed ^ 0x9e3779b9u);
    x = fmix32(x ^ (uint32_t)sample);
    x = fmix32(x ^ (uint32_t)b);
    x = fmix32(x ^ (uint32_t)h);
    return fmix32(x ^ (uint32_t)qb);
}
// The round of the search an ensemble sample perturbs, or -1 (plain mask): maxlen = longest initial node.
__device__ __forceinline__ int ens_round_of(int sample, int maxlen)
{
    if (sample <= 0) return -1;
    int rounds = 0;
    for (; maxlen > 1; maxlen = (maxlen + 1) >> 1) ++rounds;
    return rounds >> 1;
}
// The key the selection of the perturbed round compares, from the key of the branch's score (0 = empty slot).
__device__ __forceinline__ uint32_t ens_key(uint32_t key, uint32_t unit_hash, int rep_blk, float r_e)
{
    if (key == 0u) return 0u;
    const uint32_t bits = (key & 0x80000000u) ? (key ^ 0x80000000u) : ~key;  // inverse of score_key
    const uint32_t x = fmix32(unit_hash ^ (uint32_t)rep_blk);
    const float u = (float)((int)(x >> 8) - (1 << 23)) * (1.0f / 8388608.0f);   // exact
    const float moved = __fadd_rn(__uint_as_float(bits), __fmul_rn(r_e, u));    // no fused multiply-add
    return score_key(moved);
}

constexpr uint32_t kKeyNegInf = 0x007fffffu;  // score_key(-inf): a real branch without admissible pair

// rounded chunk bound round(j*Tb/kb), halves up, with Tb = a*kb + r split so that
// everything fits 32-bit arithmetic (j, r <= 1024).
__device__ __forceinline__ int chunk_bound(int j, int a, int r, int kb)
{
    return j * a + (2 * j * r + kb) / (2 * kb);
}

/*
 * Ordered top-kb selection among NB = 64*E keyed slots, run by one wave.
 *
 * Slot i*64 + lane is held by register i of `lane`.  Keeps the kb slots with the largest
 * keys (key 0 = empty slot, never kept); among equal keys the lower slot wins.  Returns for
 * each held slot whether it is kept and its rank among the kept slots in slot order, so
 * survivors can be written out compacted and still sorted by position.
 *
 * The kb-th largest key is found by a bitwise search on the key value: at most 32 steps
 * (it stops as soon as a candidate has exactly kb keys at or above it), each a compare per
 * register plus a wave ballot and a scalar popcount - no sort, no barrier.
 */
template <int E>
__device__ __forceinline__ void select_topk_ordered(const uint32_t (&key)[E], int kb, bool (&keep)[E],
                                                    int (&dest)[E])
{
    uint32_t v = 0;
#pragma unroll 1
    for (int bit = 31; bit >= 0; --bit) {
        uint32_t cand = v | (1u << bit);
        int c = 0;
#pragma unroll
        for (int i = 0; i < E; ++i) c += __popcll(__ballot(key[i] >= cand));
        if (c >= kb) v = cand;
        if (c == kb) break;  // exactly kb keys are >= cand: the kept set is settled
    }
    int c_gt = 0;
#pragma unroll
    for (int i = 0; i < E; ++i) c_gt += __popcll(__ballot(key[i] > v));
    const int need = kb - c_gt;  // how many slots equal to the threshold are still wanted
    int base_keep = 0, base_tie = 0;
#pragma unroll
    for (int i = 0; i < E; ++i) {
        bool gt = key[i] > v;
        bool eq = (key[i] == v) && (v != 0);
        uint64_t beq = __ballot(eq);
        int tie_rank = base_tie + lane_prefix_count(beq);
        bool kp = gt || (eq && tie_rank < need);
        uint64_t bkp = __ballot(kp);
        keep[i] = kp;
        dest[i] = base_keep + lane_prefix_count(bkp);
        base_tie += __popcll(beq);
        base_keep += __popcll(bkp);
    }
}

// ---- wave-local helpers -----------------------------------------------------------------

// Orders LDS traffic of ONE wave: lanes may read what other lanes of the same wave wrote
// before this point.  (LDS executes a wave's accesses in order; this only stops the compiler
// from moving them.)
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Placement of work items on the 8 XCDs (workgroup `bid` runs on XCD bid % 8, each XCD has its own L2).
// A "group" is one (sequence, kv head): everything that reads the same K/V rows.  xcd_map = 0: linear
// order.  Otherwise gc = xcd_map in {1, 2, 4, 8} groups are worked on at a time: the XCDs x with equal
// x % gc share a group (8 / gc of them, each taking every (8/gc)-th workgroup of it) and the groups are
// gone through gc at a time - few enough that the rows being read fit the memory-side cache.
// upw = work items per workgroup, unit = this wave's item inside the workgroup.  False: nothing to do.
// (32-bit arithmetic: a launch covers fewer than 2^32 work items, the launchers check; 64-bit divisions here cost
// every wave several hundred scalar instructions before it starts.)
__device__ __forceinline__ bool place_item(int xcd_map, uint32_t bid, int upw, int unit, uint32_t per_group, uint32_t groups,
                                           uint32_t &group, uint32_t &o)
{
    if (!xcd_map) {
        const uint32_t lin = bid * (uint32_t)upw + (uint32_t)unit;
        group = lin / per_group;
        o = lin - group * per_group;
        return group < groups;
    }
    // gc = xcd_map is 1, 2, 4 or 8; upw is 1 or 4
    const uint32_t lgc = (uint32_t)__builtin_ctz((uint32_t)xcd_map), ls = 3u - lgc, x = bid & 7u, q = bid >> 3;
    const uint32_t wpg = upw == 4 ? per_group >> 2 : per_group;   // workgroups per group
    const uint32_t wpp = (wpg + (1u << ls) - 1u) >> ls;            // per XCD and group
    const uint32_t qd = q / wpp, qm = q - qd * wpp;
    const uint32_t w_g = (qm << ls) + (x >> lgc);
    group = (qd << lgc) + (x & ((1u << lgc) - 1u));
    o = w_g * (uint32_t)upw + (uint32_t)unit;
    return group < groups && w_g < wpg;
}

// Host side: the launch size that goes with place_item, and how many groups to work on at a time: the largest
// power of two up to 8 with gc * bytes_per_group <= budget.  Fewer groups at a time keep the rows being read inside
// the 256 MB memory-side cache, more of them give every XCD's L2 a kv head of its own; where the balance lies was
// measured per kernel (mask estimation: 160 MB; sparse attention, which reads every gathered row once: 768 MB).
inline int64_t placed_workgroups(int xcd_map, int upw, int64_t per_group, int64_t groups)
{
    if (!xcd_map) return (groups * per_group + upw - 1) / upw;
    const int gc = xcd_map, s = 8 / gc;
    const int64_t wpg = per_group / upw, wpp = (wpg + s - 1) / s;
    return 8 * (groups / gc) * wpp;
}
inline int groups_at_a_time(int64_t bytes_per_group, int64_t budget_bytes)
{
    int gc = 8;
    while (gc > 1 && gc * bytes_per_group > budget_bytes) gc >>= 1;
    return gc;
}

template <int CTRL> __device__ __forceinline__ float dpp_f(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}

// Sum over the LPR (8 or 16) consecutive lanes that share a key row; every lane gets the sum.
template <int LPR> __device__ __forceinline__ float row_group_sum(float v)
{
    v += dpp_f<0xB1>(v);   // quad_perm [1,0,3,2]
    v += dpp_f<0x4E>(v);   // quad_perm [2,3,0,1]
    v += dpp_f<0x141>(v);  // row_half_mirror
    if (LPR == 16) v += dpp_f<0x140>(v);  // row_mirror
    return v;
}

// fp32 dot product of two runs of 8 bf16 values (v_dot2_f32_bf16 x 4).
__device__ __forceinline__ float dot8_bf16(const uint4 &a, const uint4 &b)
{
    typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
    float acc = 0.f;
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.x), __builtin_bit_cast(bf16x2_t, b.x), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.y), __builtin_bit_cast(bf16x2_t, b.y), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.z), __builtin_bit_cast(bf16x2_t, b.z), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.w), __builtin_bit_cast(bf16x2_t, b.w), acc, false);
    return acc;
}

}  // namespace hipattn
