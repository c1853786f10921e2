/*
 * hipattn - Hierarchically Pruned Attention (HiP) hot path for AMD MI355X (gfx950).
 *
 * C ABI of the two operations of the paper's problem statement:
 *
 *   hip_mask_estimate : hierarchical top-k key estimation
 *                       (paper Sec. 3.1 "Hierarchical Score-Locality-Aware Top-k Estimation",
 *                        Sec. 3.2 "Block Approximation", Alg. 1; per-step use in Alg. 2)
 *   hip_sparse_attn   : block-sparse attention over the selected keys
 *                       (paper Eq. 1-3; "Block Sparse Flash Attention" in the appendix)
 *
 * NOTE ON NAMES: "hip_" / "HIP_" here abbreviates the method (HiP attention), not the
 * GPU runtime whose symbols are spelled hipXxx.
 *
 * General rules for every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library never
 *     allocates, frees, copies to the host or synchronises; a call validates its
 *     arguments on the host and enqueues kernels on `stream` (a hipStream_t passed as
 *     void*; NULL = the default stream).  Results are ready when the stream reaches them.
 *   - `hip_problem` itself is read on the host during the call and may be freed afterwards;
 *     the arrays it points to (kv_lens, page_table) are DEVICE arrays read by the kernels.
 *   - Return value: HIP_ATTN_OK (0), a negative HIP_ATTN_E* argument error detected before
 *     any launch, or HIP_ATTN_ELAUNCH - (hipError_t) for a failed launch.  Nothing is
 *     printed; NaN/Inf inputs give unspecified indices.
 *   - Re-entrant; no mutable global state, except for hip_mask_estimate_noalloc (its static scratch, see there).
 *
 * Conventions (0-based):
 *   kb      = k / bk                       key blocks kept per query block
 *   g       = n_q_heads / n_kv_heads       query head h reads KV head h / g
 *   pos(i)  = kv_len - q_len + i           absolute position of query row i of a sequence
 *   query block qb = rows [qb*bq, min((qb+1)*bq, q_len)); it searches the key blocks of
 *   its visible prefix [0, min(kv_len, pos(last row)+1)).
 */
#ifndef HIPATTN_H
#define HIPATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HIP_ATTN_SENTINEL INT32_MAX /* "no block" entry of the index array */

enum {
    HIP_ATTN_OK = 0,
    HIP_ATTN_ENULL = -1,       /* a required pointer is NULL                                  */
    HIP_ATTN_ESHAPE = -2,      /* non-positive size, n_q_heads % n_kv_heads, q_len > kv_len,  */
                               /* negative n_sink / n_window / top_r                          */
    HIP_ATTN_EBLOCK = -3,      /* k % bk != 0, bq/bk out of range, b_sq > bq, bk % b_sk != 0, */
                               /* unknown rep_pos                                             */
    HIP_ATTN_EHEADDIM = -4,    /* head_dim not in {64, 128}                                   */
    HIP_ATTN_EDTYPE = -5,      /* dtype not HIP_ATTN_F32 / HIP_ATTN_BF16                      */
    HIP_ATTN_ETOOLARGE = -6,   /* k/bk above HIP_ATTN_MAX_KB, or bq*head_dim above the limit  */
    HIP_ATTN_EALIGN = -7,      /* a pointer or row stride is not 16-byte aligned              */
    HIP_ATTN_EPAGE = -8,       /* page table given with page_size <= 0 or page_size % bk != 0; a backing   */
                               /* pool or a touched map without a page table                   */
    HIP_ATTN_EWORKSPACE = -9,  /* workspace_bytes below hip_workspace_bytes()                 */
    HIP_ATTN_EENSEMBLE = -11,  /* n_e, theta_vote or n_e * k/bk out of range                              */
    HIP_ATTN_ESCRATCH = -10,   /* hip_mask_estimate_noalloc: hip_workspace_bytes() above the static scratch */
    HIP_ATTN_ELAUNCH = -1000   /* launch failure: code is HIP_ATTN_ELAUNCH - hipError_t       */
};

enum { HIP_ATTN_F32 = 0, HIP_ATTN_BF16 = 1 };
enum { HIP_ATTN_REP_CENTER = 0, HIP_ATTN_REP_FIRST = 1, HIP_ATTN_REP_LAST = 2 };

/* flags */
enum {
    HIP_ATTN_FORCE_GENERIC = 1, /* use the shape-generic kernels even where a tuned one exists */
    HIP_ATTN_NO_SHARED_ROUND = 2 /* prefill mask estimation: every head gathers the first round's key tiles itself, */
                                 /* even where the heads of a KV group could share them (A/B measurements)          */
};

#define HIP_ATTN_MAX_KB 1024   /* largest k/bk                                                */
#define HIP_ATTN_MAX_BQ 64     /* largest query block                                         */
#define HIP_ATTN_MAX_BK 16     /* largest key block                                           */

typedef struct hip_problem {
    int32_t batch, n_q_heads, n_kv_heads, head_dim; /* head_dim in {64,128}                     */
    int32_t q_len;       /* query rows per sequence: T for prefill, 1 for decode (bq is then    */
                         /* taken as 1: the single row is its own query block)                 */
    int32_t max_kv_len;  /* T of contiguous K/V, or the largest kv_lens[b]                     */
    int32_t k, bq, bk;   /* k % bk == 0; 1 <= bq <= 64; 1 <= bk <= 16                          */
    int32_t dtype;       /* HIP_ATTN_F32 or HIP_ATTN_BF16; Q, K, V, O all have this type       */
    int32_t flags;       /* HIP_ATTN_FORCE_GENERIC or 0                                        */
    float sm_scale;      /* softmax scale of hip_sparse_attn; <= 0 selects 1/sqrt(head_dim)    */
    const int32_t *kv_lens;    /* device [batch], q_len <= kv_lens[b] <= max_kv_len; NULL = max_kv_len */
    const int32_t *page_table; /* device [batch, max_pages] or NULL (contiguous K/V)           */
    int32_t page_size, max_pages; /* tokens per page (multiple of bk); row length of the table */
    /* Element strides (batch, head, row); the channel dimension is contiguous.  All zero =
     * dense row-major: Q,O [batch, n_q_heads, q_len, head_dim]; K,V [batch, n_kv_heads,
     * max_kv_len, head_dim], or with a page table the pool [n_pages, n_kv_heads, page_size,
     * head_dim] where kv_strides[0] is the page stride.  Row strides must keep rows 16-byte
     * aligned. */
    int64_t q_strides[3], kv_strides[3], o_strides[3];
    /* hip_sparse_attn only (paper appendix "Block Sparse Flash Attention": a global sink and a small
     * sliding window are attended in addition to the selected blocks): every row also attends to the
     * first n_sink keys and to the n_window most recent keys up to its own position; each key counts
     * once.  0 = off.  With a window that covers the steps since the last hip_mask_estimate call, an
     * index array from an earlier (shorter) kv_len may be reused as is (Alg. 2, mask refresh period). */
    int32_t n_sink, n_window;
    /* hip_mask_estimate only: the block score may be taken over a sample of the query block's rows
     * and of the representative block's keys (paper Sec. 3.2, last paragraph): rows 0, b_sq, 2*b_sq, ...
     * and keys 0, b_sk, 2*b_sk, ... of the block.  0 or 1 = every row / key.  b_sk must divide bk.
     * A non-empty branch none of whose sampled (row, key) pairs is admissible scores -inf (it still
     * outranks an empty branch). */
    int32_t b_sq, b_sk;
    /* hip_mask_estimate only: which block of a branch represents it: HIP_ATTN_REP_CENTER (default,
     * paper Sec. 3.1), _FIRST or _LAST (the paper's appendix ablates the position). */
    int32_t rep_pos;
    /* hip_mask_estimate only: top-r approximation of the scores (paper appendix "Top-r Approximation"):
     * the products of a query row run over the top_r channels in which that row's |q| is largest (the
     * lower channel among equal magnitudes); each row of a query block has its own channel set.
     * 0 or >= head_dim = all channels (the default of the paper).  The call first writes a copy of Q
     * with the other channels zeroed into `workspace` and estimates the mask from that copy: a row's
     * channels are scattered over every 32-byte sector of a key row, so whole key rows are still
     * fetched on this hardware and the option serves accuracy studies, not speed. */
    int32_t top_r;
    /* Device scratch owned by the caller, 16-byte aligned, at least hip_workspace_bytes(p) bytes; read and
     * written by the call's kernels only, free for reuse once the stream has passed them.  May be NULL
     * when hip_workspace_bytes(p) is 0 (every problem without top_r). */
    void *workspace;
    size_t workspace_bytes;
    /* Token bank with a vector-map page table (paper Sec. 3.3, "KV Token Index Translation"): with a page
     * table, K (and V) is the pool of GPU-resident pages (the bank) and an entry e >= 0 of the table names
     * page e of it, as always.  An entry e < 0 is a miss: the page is read from page ~e (= -e - 1) of the
     * backing pool k_backing / v_backing instead, any memory the GPU can read (device memory, or pinned host
     * memory for an offloaded cache), laid out and strided exactly like K / V.  hip_mask_estimate reads
     * k_backing only; hip_sparse_attn both.  NULL = the table holds no negative entry (a negative entry is
     * then undefined behaviour).  Each call has its own problem description, so mask estimation and sparse
     * attention can use different banks and tables, as the paper's two offloading contexts do. */
    const void *k_backing, *v_backing;
    /* Device [batch, max_pages] bytes or NULL; needs a page table.  The call stores 1 at (b, i) for every
     * logical page i of sequence b that it reads a key of: hip_mask_estimate the pages of the representative
     * blocks it scores (any head, any query block, any round), hip_sparse_attn the pages of the keys its
     * rows attend to (selected blocks visible to a row of their query block, sink, window).  Other bytes are
     * left as they are, so the caller zeroes the map and may let it accumulate over calls: it is what a
     * cache manager needs to count hits and misses (compare with the table) and to pick the pages to load. */
    uint8_t *touched;
    /* hip_mask_estimate only: ensemble sample (paper appendix "Ensemble Hierarchical Top-k Approximation": several
     * masks are drawn "by adding randomness r_e to the branch direction" of a middle iteration, then voted on).
     * ens_sample = 0 (default) is the plain mask.  A sample e > 0 differs in one round of the search, round
     * R / 2 of the R = ceil(log2(ceil(Tb / (k/bk)))) rounds of a query block with Tb visible key blocks (rounds
     * counted from 0): there the top-k selection compares score + ens_r * u instead of the score, u a draw on
     * [-1, 1) fixed by (ens_seed, e, sequence, head, query block, representative block): the 32-bit finalizer of
     * MurmurHash3, x ^= x >> 16; x *= 0x85ebca6b; x ^= x >> 13; x *= 0xc2b2ae35; x ^= x >> 16, is applied to
     * ens_seed ^ 0x9e3779b9 and then, five times, to (previous result ^ next number); with n the top 24 bits of
     * the last result, u = (n - 2^23) / 2^23.  Product and sum are single precision, each rounded once. */
    int32_t ens_sample;
    uint32_t ens_seed;
    float ens_r;
} hip_problem;

/*
 * Hierarchical mask estimation (Alg. 1 with the block form of Sec. 3.2).
 *   Q        device, layout per q_strides
 *   K        device, layout per kv_strides (sequence-major, or the page pool)
 *   indices  device int32 [batch, n_q_heads, ceil(q_len/bq), k/bk], written by the call:
 *            row (b,h,qb,:) holds the first logical token position (a multiple of bk) of each
 *            selected key block, strictly ascending, followed by HIP_ATTN_SENTINEL padding
 *            when fewer than k/bk blocks are visible.  Positions are logical (before page
 *            translation).
 * Scores are unscaled dot products accumulated in fp32; the score of a branch is the maximum
 * over the query block's rows and the representative (centre) key block's keys of the
 * causally admissible products; equal scores are resolved towards the lower position.
 */
int hip_mask_estimate(const hip_problem *p, const void *Q, const void *K, int32_t *indices,
                      void *stream);

/*
 * Block-sparse attention (Eq. 2-3 with the mask given by `indices`).
 *   indices  as written by hip_mask_estimate; any entry < 0 or >= kv_len means "no block";
 *            valid entries of a row must be distinct.
 *   O        device, layout per o_strides, same dtype as Q.  Row i attends to the keys t of
 *            its query block's selected blocks (plus sink and window keys, see hip_problem) with
 *            t < kv_len and t <= pos(i); a row with no such key is written as zeros.  Softmax
 *            statistics and accumulation are fp32.
 */
int hip_sparse_attn(const hip_problem *p, const void *Q, const void *K, const void *V,
                    const int32_t *indices, void *O, void *stream);

/* Device scratch hip_mask_estimate needs for this problem: one copy of Q when top_r is in use,
 * otherwise 0 (the kernels keep their state in LDS and registers).  hip_sparse_attn needs none. */
size_t hip_workspace_bytes(const hip_problem *p);

/*
 * hip_mask_estimate for callers that cannot allocate device memory or hand over a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments, results and errors as
 * hip_mask_estimate, except that p->workspace / p->workspace_bytes are ignored: the scratch the top_r option
 * needs (hip_workspace_bytes(p) bytes) is a static array of HIP_ATTN_STATIC_SCRATCH_BYTES inside the library,
 * one copy per GPU, held until the process ends.  A problem that needs more returns HIP_ATTN_ESCRATCH before any
 * launch.  The call allocates and frees nothing.  Every call on a GPU shares that GPU's array (it keeps the last
 * call's contents; the call overwrites what it reads): calls that overlap in time on one GPU - different streams,
 * or different host threads - race on it and must be serialised by the caller.
 */
#define HIP_ATTN_STATIC_SCRATCH_BYTES (8u << 20)
int hip_mask_estimate_noalloc(const hip_problem *p, const void *Q, const void *K, int32_t *indices,
                              void *stream);

/*
 * Vote over an ensemble of masks (paper appendix "Ensemble Hierarchical Top-k Approximation", second step).
 *   samples  device int32 [n_e][batch, n_q_heads, ceil(q_len/bq), k/bk]: n_e index arrays as hip_mask_estimate
 *            writes them (every row ascending, then HIP_ATTN_SENTINEL padding; entries < 0 count as padding)
 *   indices  device int32 [batch, n_q_heads, ceil(q_len/bq), width], width = k/bk if tau else n_e * k/bk:
 *            per query block the positions held by at least theta_vote of the n_e rows (1 = union, n_e =
 *            intersection), ascending, HIP_ATTN_SENTINEL-padded.  tau = 1 keeps at most k/bk of them: those with
 *            more votes first, the lower position among equal votes.
 * Only batch, n_q_heads, q_len, bq, k, bk of `p` are used.  1 <= n_e <= 16, n_e * k/bk <= 4096, 1 <= theta_vote.
 * hip_sparse_attn takes the result with k set to width * bk (so width must stay within HIP_ATTN_MAX_KB).
 */
int hip_mask_vote(const hip_problem *p, const int32_t *samples, int32_t n_e, int32_t theta_vote, int32_t tau,
                  int32_t *indices, void *stream);

/*
 * Ensemble mask in one call: samples 0 .. n_e - 1 of hip_mask_estimate (p->ens_sample is ignored; p->ens_seed
 * and p->ens_r apply; sample 0 is the plain mask) into p->workspace, then hip_mask_vote into `indices`.
 * p->workspace must hold hip_ensemble_workspace_bytes(p, n_e) bytes, 256-byte aligned: the n_e index arrays,
 * after the scratch of the top_r option when that is in use.
 */
int hip_mask_ensemble(const hip_problem *p, const void *Q, const void *K, int32_t n_e, int32_t theta_vote,
                      int32_t tau, int32_t *indices, void *stream);
size_t hip_ensemble_workspace_bytes(const hip_problem *p, int32_t n_e);

/* Static, human-readable text for a return code. */
const char *hip_strerror(int code);

/* Library version, major*100 + minor. */
int hip_attn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* HIPATTN_H */
