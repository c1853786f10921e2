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
    int64_t qs_b, qs_h, qs_r;  // element strides
    int64_t ks_b, ks_h, ks_r;
    int64_t os_b, os_h, os_r;
    int32_t batch, hq, hkv, g, d, q_len, max_kv_len, kb, bq, bk, nqb, page_size, max_pages;
    float sm_scale;
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

// Element offset of logical key/value row t of sequence b, kv head h.
__device__ __forceinline__ int64_t kv_row_offset(const KParams &p, int b, int h, int t)
{
    if (p.page_table) {
        int pg = p.page_table[(int64_t)b * p.max_pages + t / p.page_size];
        return (int64_t)pg * p.ks_b + (int64_t)h * p.ks_h + (int64_t)(t % p.page_size) * p.ks_r;
    }
    return (int64_t)b * p.ks_b + (int64_t)h * p.ks_h + (int64_t)t * p.ks_r;
}

__device__ __forceinline__ int lane_prefix_count(uint64_t mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}

// rounded chunk bound round(j*Tb/kb), halves up, with Tb = a*kb + r split so that
// everything fits 32-bit arithmetic (j, r <= 1024).
__device__ __forceinline__ int chunk_bound(int j, int a, int r, int kb)
{
    return j * a + (2 * j * r + kb) / (2 * kb);
}

/*
 * Ordered top-kb selection among NB = 64*E keyed slots, run redundantly by every wave.
 *
 * Slot i*64 + lane is held by register i of `lane`.  Keeps the kb slots with the largest
 * keys (key 0 = empty slot, never kept); among equal keys the lower slot wins.  Returns for
 * each held slot whether it is kept and its rank among the kept slots in slot order, so
 * survivors can be written out compacted and still sorted by position.
 *
 * The kb-th largest key is found by a bitwise search on the key value: 32 steps, each a
 * compare per register plus a wave ballot and a scalar popcount - no sort, no barrier.
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

}  // namespace hipattn
