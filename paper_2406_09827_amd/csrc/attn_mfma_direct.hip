// Block-sparse attention for bf16 prefill at head dim 128 on CDNA4 matrix cores (paper Eq. 2-3; the "block
// sparse flash attention" of the appendix), with the gathered key and value rows loaded STRAIGHT INTO LDS.
//
// Same work split and arithmetic as attn_mfma.hip (one wave = one 32-row query tile of one (sequence, head, query
// block); per tile of 32 gathered keys S^T = K Q^T, lane-local online softmax, O^T += V^T P^T with the value
// tile read back channel-major by ds_read_b64_tr_b16).  What differs is how a tile travels: the counters of the
// register-staged kernel showed the LDS instruction pipe 91 % busy (16 ds_write_b128 + 24 reads per tile) with the
// matrix pipe at 21 %, so here
//   * global_load_lds_dwordx4 delivers lane l's 16 bytes at M0 + 16 l without passing through registers or the LDS
//     instruction pipe: load j of a tile fills LDS rows 4j .. 4j+3; lane group lg = l / 16 supplies gathered key
//     8 lg + j (a lane's 8 rows are consecutive keys, so one 16-byte LDS read tells it where they are), hence key x
//     sits in LDS row 4 (x % 8) + x / 8; the XOR swizzles that keep the operand reads free of bank conflicts are
//     applied to the global chunk a lane fetches (keys: 16-byte chunk c at place c ^ (x % 16); values: 32-byte
//     chunk pair p at place p ^ rotl3(x % 8), so that the 16 consecutive channels a transpose read takes stay together
//     and the eight 32-byte pieces that 32 lanes of a transpose read fetch fall into different banks);
//   * the LDS is a pure staging area with ONE key and ONE value buffer per wave: as soon as a tile's key operands
//     are in registers the key buffer is refilled with the next tile's keys, which land while this tile is
//     multiplied and its softmax runs; the same for the values after the transpose reads;
//   * the direct loads are inline assembly with hand-placed waits (the compiler neither knows that they write LDS
//     nor counts them) and they are the only vector memory instructions of the loop: a compiler-visible load in
//     there would make the compiler wait for all of them.  The work item's row of the index array is therefore
//     copied into LDS once, before the loop.
//   * P is a single bf16 term; the row sum is taken over the ROUNDED probabilities, so numerator and denominator of
//     the output carry the same weights.
// The wave raises its priority while it feeds the matrix pipe, so that of the two waves of a SIMD one multiplies
// while the other runs its softmax arithmetic.
#include "common.h"
#include "launch.h"

namespace hipattn {

namespace {

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

constexpr int D = 128;
constexpr int KS = D / 16;      // k-steps of S^T = K Q^T
constexpr int CT = D / 32;      // 32-channel tiles of O^T
constexpr int NLD = 8;          // wave-wide 16-byte loads per 32-row tile (4 rows of 256 bytes each)
constexpr int ROWB = D * 2;     // bytes per row
constexpr int TILEB = 32 * ROWB;
// LDS of a workgroup, carved by hand so that the tile buffers (the targets of the direct loads, whose LDS address
// travels in M0) lie in the first 64 KB:
constexpr int kOffK = 0, kOffV = 4 * TILEB, kOffTk = 8 * TILEB, kOffMo = kOffTk + 4 * 3 * 32 * 4, kOffMl = kOffMo + 4 * 2 * 32 * 4;
constexpr int kOffIdx = kOffMl + 4 * 2 * 64 * 4;   // the work items' rows of the index array follow
static_assert(kOffTk <= 65536, "direct-load targets must stay below 64 KB");

}  // namespace

// MODE 0: contiguous K/V, a (sequence, kv head) slice below 4 GB: rows are addressed by a scalar slice base plus a
//         32-bit lane offset; MODE 1: paged pool; MODE 2: contiguous, any size (64-bit row addresses).
// SPLIT: the workgroup takes ONE work item; wave w walks key tiles w, w + 4, ... with its own softmax state and the
//        four states are merged through LDS at the end (for launches with too few work items to fill the GPU).
// CAP: index entries (k/bk) a work item may have; with 512 two workgroups share a compute unit, with 1024 one.
template <int MODE, bool SPLIT, int CAP>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2))) void attn_mfma_direct_kernel(KParams p, int log_bk, int mtn, int xcd_map)
{
    constexpr bool PAGED = MODE == 1, A32 = MODE == 0;
    __shared__ __attribute__((aligned(1024))) char lds[kOffIdx + (SPLIT ? 1 : 4) * CAP * 4];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, hh = lane >> 5;
    const int lg = lane >> 4, lc = lane & 15;  // loading role: gathered keys lg*8 .. lg*8+7, LDS chunk place lc

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

    auto uniform64 = [](int64_t v) __attribute__((always_inline)) {
        return ((int64_t)__builtin_amdgcn_readfirstlane((int)(v >> 32)) << 32) | (uint32_t)__builtin_amdgcn_readfirstlane((int)v);
    };
    const bf16_t *Kbase = (const bf16_t *)p.K, *Vbase = (const bf16_t *)p.V;
    const int64_t seq_off = (int64_t)b * p.ks_b + (int64_t)hk * p.ks_h;  // contiguous layout: row 0 of this slice
    // the same in every lane: as a scalar it becomes the scalar base of the row loads
    const int64_t slice_u = uniform64(seq_off * 2);
    const char *Kseq = (const char *)p.K + slice_u, *Vseq = (const char *)p.V + slice_u;
    // this work item's row of the index array, copied into LDS (with SPLIT the four waves write the same values)
    int *idxs = (int *)(lds + kOffIdx) + (SPLIT ? 0 : wave) * CAP;
    {
        const int32_t *idx = p.idx_in + (((int64_t)b * p.hq + h) * p.nqb + qb) * p.kb;
        for (int j = lane; j < p.kb; j += 64) idxs[j] = idx[j];
    }

    char *kt = lds + kOffK + wave * TILEB, *vt = lds + kOffV + wave * TILEB;
    // per tile, published two tiles ahead: key positions (three slots: the tile being masked and the two published ones)
    // and row offsets (two slots)
    int *tk_base = (int *)(lds + kOffTk) + wave * 96;
    uint32_t *mo_base = (uint32_t *)(lds + kOffMo) + wave * 64;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)lds;
    const uint32_t kt_m0 = lds0 + kOffK + wave * TILEB, vt_m0 = lds0 + kOffV + wave * TILEB;

    const float c = p.sm_scale * 1.44269504088896340736f;  // scores are kept in log2 units
    constexpr float kSlack = 8.f;
    float m_run = -INFINITY, l_run = 0.f;
    f32x16 oacc[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[ct][r] = 0.f;

    // this wave's tiles: all of them, or every fourth one (SPLIT)
    const int nt = SPLIT ? (n_tiles > wave ? (n_tiles - wave + 3) >> 2 : 0) : n_tiles;
    auto tile_of = [&](int i) __attribute__((always_inline)) { return SPLIT ? wave + 4 * i : i; };

    // Metadata of a tile of 32 gathered keys: lane `col` works out key `col` (position or -1, and what a loading
    // lane needs to find the row) and publishes both.  Rows that do not count load row 0 of the sequence (always
    // mapped, finite) and get probability 0.  Returns flags: bit 0 = some key may count for some row, bit 1 = some
    // (key, row) pair needs masking, bit 2 = window tile.
    auto publish_tile = [&](int tile, int *tk, uint32_t *mo) __attribute__((always_inline)) {
        int t_c = -1;
        int flags;
        if (tile < tiles_sel) {
            const int ki = tile * 32 + col;
            if (ki < n_keys) {
                const int first = idxs[ki >> log_bk];
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
        const int tr = t_c >= 0 ? t_c : 0;
        // the page (paged pool) or the row's offset from the start of this sequence / kv head slice in 16-byte units
        const uint32_t m = PAGED ? (uint32_t)page_of_row<true>(p, b, tr) : (uint32_t)(((int64_t)tr * p.ks_r) >> 3);
        if (hh == 0) {
            tk[col] = t_c;
            mo[col] = m;
        }
        return flags;
    };
    // Where this lane's 8 rows of the published tile are: offsets (or pages) and, for a paged pool, positions.
    struct rows_t { uint32_t off[NLD]; int tkl[PAGED ? NLD : 1]; };
    auto read_rows = [&](const int *tk, const uint32_t *mo, rows_t &R) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < NLD; j += 4) {
            const uint4 m4 = *(const uint4 *)(mo + lg * NLD + j);
            R.off[j] = m4.x; R.off[j + 1] = m4.y; R.off[j + 2] = m4.z; R.off[j + 3] = m4.w;
        }
        if (PAGED) {
#pragma unroll
            for (int j = 0; j < NLD; j += 4) {
                const int4 t4 = *(const int4 *)(tk + lg * NLD + j);
                R.tkl[j] = t4.x; R.tkl[j + 1] = t4.y; R.tkl[j + 2] = t4.z; R.tkl[j + 3] = t4.w;
            }
        }
    };
    // The 8 direct loads of a tile's keys (VAL = false) or values (VAL = true): load j brings gathered key x = 8 lg + j
    // to LDS row 4 j + lg, this lane the 16-byte chunk that belongs at place lc of that row.  (M0 is a reserved
    // register: the compiler warns that it does not track the clobber.  It is written and consumed inside one asm
    // statement, and nothing else in this kernel uses M0.)
    auto issue_rows = [&](const rows_t &R, bool val) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
            const int x = lg * NLD + j;
            const int rot = ((x & 3) << 1) | ((x >> 2) & 1);   // x % 8 rotated left by one bit
            const uint32_t chunk = val ? (uint32_t)(((((lc >> 1) ^ rot) << 1) | (lc & 1)) << 4) : (uint32_t)((lc ^ (x & 15)) << 4);
            const uint32_t dst = __builtin_amdgcn_readfirstlane((val ? vt_m0 : kt_m0) + j * 1024);
            if (A32) {
                const uint32_t vo = (R.off[j] << 4) + chunk;
                const char *base = val ? Vseq : Kseq;
                asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                             :: "v"(vo), "s"(base), "s"(dst) : "memory", "m0");
            } else {
                const char *src;
                if (PAGED) {
                    // (a negative page-table entry names a page of the backing pools)
                    const int tr = max(R.tkl[j], 0), e = (int)R.off[j];
                    const bf16_t *pool = (const bf16_t *)(val ? pool_of(e, Vbase, p.Vback) : pool_of(e, Kbase, p.Kback));
                    src = (const char *)(pool + row_offset_in<true>(p, b, hk, tr, page_in_pool(e))) + chunk;
                } else {
                    src = (const char *)((val ? Vbase : Kbase) + seq_off + ((int64_t)R.off[j] << 3)) + chunk;
                }
                asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                             :: "v"(src), "s"(dst) : "memory", "m0");
            }
        }
    };

    // The query loads end here, where the compiler can see it: it does not count the loads that the loop issues from
    // inline assembly, and a wait for a query fragment left inside that loop would wait for them.
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) asm volatile("" :: "v"(qf[kk]));

    // Outstanding vector memory operations at the top of iteration i, oldest first: keys of tile i (8), values of
    // tile i (8).
    int flags_cur = 0, flags_nxt = 0;
    int *tk0 = tk_base, *tk1 = tk_base + 32, *tk2 = tk_base + 64;   // slots of tiles i, i+1, i+2
    wave_lds_sync();   // the index row is in LDS
    if (nt > 0) {
        rows_t R0;
        flags_cur = publish_tile(tile_of(0), tk0, mo_base);
        if (nt > 1) flags_nxt = publish_tile(tile_of(1), tk1, mo_base + 32);
        wave_lds_sync();
        read_rows(tk0, mo_base, R0);
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");   // nothing of the compiler's is in flight from here on
        issue_rows(R0, false);
        issue_rows(R0, true);
    }
    for (int i = 0; i < nt; ++i) {
        const int flags = flags_cur;
        const bool more = i + 1 < nt;
        const int *tk = tk0;
        // ---- keys of tile i have landed; its values may still be on their way
        asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        uint4 kv[KS];
        if (flags & 1) {
            // key x = col sits in LDS row 4 (col % 8) + col / 8, chunk c at place c ^ (col % 16)
            const char *krow = kt + (4 * (col & 7) + (col >> 3)) * ROWB;
#pragma unroll
            for (int kk = 0; kk < KS; ++kk) kv[kk] = *(const uint4 *)(krow + (((kk * 2 + hh) ^ (col & 15)) << 4));
        }
        // this lane's rows of the next tile were published an iteration ago: their read rides along with the operand
        // reads, and the tile after it is published now, off the path to the next loads
        rows_t R1;
        if (more) read_rows(tk1, mo_base + ((i + 1) & 1) * 32, R1);
        int flags_2 = 0;
        if (i + 2 < nt) flags_2 = publish_tile(tile_of(i + 2), tk2, mo_base + (i & 1) * 32);
        // the key operands are in registers (and this lane's rows of the next tile are known): the key buffer may be refilled
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        if (more) issue_rows(R1, false);
        // outstanding now: values of tile i (8) [, keys of tile i+1 (8)]

        f32x16 sacc;
        bf16x8 pb[2];
        if (flags & 1) {
            // ---- S^T = K Q^T: A = key rows (lane: key col), B = queries
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
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
            // P^T as B operand of the two 16-key steps (registers 8*st .. 8*st+7), rounded to bf16; the row sum runs
            // over the rounded values (v_dot2_f32_bf16 against ones, fp32 accumulation)
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
        }

        // ---- the values of tile i have landed
        if (more) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        bf16x8 va[2][CT];
        if (flags & 1) {
            // Value tile read back channel-major with the LDS transpose read.  ds_read_b64_tr_b16 works on blocks of
            // 16 lanes: lanes 4e .. 4e+3 of a block point at 16 consecutive bf16 of source row e (e = 0..3), and lane
            // i of the block receives element i of each of the four rows.  Block = (channel half cb, key half hh):
            // rows are 4 consecutive keys, so a lane ends up with 4 keys of its channel - half an A operand per
            // read.  Key x = 16 st [+ 8] + 4 hh + e sits in LDS row 4 (4 hh + e) + 2 st [+ 1]; the 32-byte pair
            // ct*2 + cb of its channels at place (ct*2 + cb) ^ (2 e + hh).
            const int i16 = lane & 15, cb = (lane >> 4) & 1, e = i16 >> 2, x7 = 4 * hh + e;
            const char *vrow = vt + (4 * x7) * ROWB + (i16 & 3) * 8;
#pragma unroll
            for (int st = 0; st < 2; ++st)
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) {
                    const int place = ((ct * 2 + cb) ^ (2 * e + hh)) << 5;   // x7 rotated left by one bit
                    const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(vrow + (2 * st) * ROWB + place));
                    const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(vrow + (2 * st + 1) * ROWB + place));
                    const uint2 a = __builtin_bit_cast(uint2, lo4), c2 = __builtin_bit_cast(uint2, hi4);
                    va[st][ct] = __builtin_bit_cast(bf16x8, make_uint4(a.x, a.y, c2.x, c2.y));
                }
        }
        // the value operands are in registers: the value buffer may be refilled
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        if (more) issue_rows(R1, true);
        if (flags & 1) {
            // ---- O^T += V^T P^T (the CT accumulators are independent)
            __builtin_amdgcn_s_setprio(2);
#pragma unroll
            for (int st = 0; st < 2; ++st)
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) oacc[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[st][ct], pb[st], oacc[ct], 0, 0, 0);
            __builtin_amdgcn_s_setprio(0);
        }
        flags_cur = flags_nxt; flags_nxt = flags_2;
        { int *t = tk0; tk0 = tk1; tk1 = tk2; tk2 = t; }
    }

    if (SPLIT) {
        // Waves 1-3 leave their state (running reference, partial sum, accumulators) in their own tile buffers,
        // lane-contiguous; wave 0 folds them into its own: with m = max of the references, every state is rescaled
        // by 2^(m_w - m) before it is added (the usual merge of online-softmax states).
        float *sk = (float *)kt, *sv = (float *)vt, *ml = (float *)(lds + kOffMl) + wave * 128;
        if (wave != 0) {
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float *dst = ct < CT / 2 ? sk + (ct * 16 + r) * 64 : sv + ((ct - CT / 2) * 16 + r) * 64;
                    dst[lane] = oacc[ct][r];
                }
            ml[lane] = m_run;
            ml[64 + lane] = l_run;
        }
        __syncthreads();
        if (wave != 0) return;
#pragma unroll
        for (int w = 1; w < 4; ++w) {
            const float *ok = (const float *)(lds + kOffK + w * TILEB), *ov = (const float *)(lds + kOffV + w * TILEB);
            const float *mlw = (const float *)(lds + kOffMl) + w * 128;
            const float m_w = mlw[lane], l_w = mlw[64 + lane];
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

    // ---- normalise, transpose through LDS (16-byte chunk c of row r at place c ^ (r % 16)), coalesced store
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            uint2 u;
            u.x = pack_bf16(oacc[ct][4 * g + 0] * inv, oacc[ct][4 * g + 1] * inv);
            u.y = pack_bf16(oacc[ct][4 * g + 2] * inv, oacc[ct][4 * g + 3] * inv);
            *(uint2 *)(vt + col * ROWB + (((ct * 4 + g) ^ (col & 15)) << 4) + hh * 8) = u;
        }
    wave_lds_sync();
    bf16_t *Ob = (bf16_t *)p.O + (int64_t)b * p.os_b + (int64_t)h * p.os_h + (int64_t)row0 * p.os_r;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int row = lg + i * 4;
        if (row < n_rows) *(uint4 *)(Ob + (int64_t)row * p.os_r + lc * 8) = *(const uint4 *)(vt + row * ROWB + ((lc ^ (row & 15)) << 4));
    }
}

// head dim 128 and k/bk <= 1024 (checked by the caller)
hipError_t launch_attn_mfma_direct(const KParams &p, dim3 grid, int log_bk, int mtn, int xcd_map, int mode, bool split, hipStream_t st)
{
    dim3 block(kThreads);
#define HIPATTN_LAUNCH(SP, CAPV)                                                                                        \
    do {                                                                                                          \
        if (mode == 1) hipLaunchKernelGGL((attn_mfma_direct_kernel<1, SP, CAPV>), grid, block, 0, st, p, log_bk, mtn, xcd_map);      \
        else if (mode == 0) hipLaunchKernelGGL((attn_mfma_direct_kernel<0, SP, CAPV>), grid, block, 0, st, p, log_bk, mtn, xcd_map); \
        else hipLaunchKernelGGL((attn_mfma_direct_kernel<2, SP, CAPV>), grid, block, 0, st, p, log_bk, mtn, xcd_map);                \
    } while (0)
    if (split) HIPATTN_LAUNCH(true, 1024);
    else if (p.kb <= 512) HIPATTN_LAUNCH(false, 512);
    else HIPATTN_LAUNCH(false, 1024);
#undef HIPATTN_LAUNCH
    return hipGetLastError();
}

}  // namespace hipattn
