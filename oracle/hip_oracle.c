/*
 * CPU oracle for Hierarchically Pruned Attention (HiP): hierarchical top-k mask
 * estimation (paper Sec. 3.1, Sec. 3.2, Alg. 1, Eq. 4-5) and top-k masked
 * attention (Eq. 1-3), plus the per-step decode use of both (Alg. 2).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, double-precision
 * restatement of what the method computes, meant to be checked against the
 * paper by eye.  Only tests, the smoke check and the benchmark's CPU-baseline
 * leg may call it; the GPU library shares no code, header, table or helper
 * with this file and never falls back to it.
 *
 * Conventions (0-based, half-open block ranges [s,e)):
 *   kb        = k / bk        number of key blocks kept per query block
 *   pos(i)    = kv_len - q_len + i   absolute position of query row i
 *   query head h reads KV head h / (n_q_heads / n_kv_heads)
 * Inputs are float arrays that already hold the dtype-rounded values (a bf16
 * value is exactly representable as a float); every sum is taken in double.
 *
 * Pins (tests/test_oracle_*.py): dense causal attention when k >= T; a fixed-depth
 * search over explicit sets of key blocks enumerated on tiny T; monotone-score
 * closed form; kb = 1 greedy binary search; the T=4k,k=512,bq=32,bk=2 structure
 * the paper prints (initial group of 8 blocks, 3 effective rounds); invariants.
 * The numeric VALUES of indices on random data have no printed example in the
 * paper: for those the oracle is pinned only by the brute-force set search
 * and the stated readings ("parity unpinned" by a paper-printed value).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_SENTINEL INT32_MAX

/* ------------------------------------------------------------------------ */
/* problem description                                                       */
/* ------------------------------------------------------------------------ */

typedef struct {
    int32_t batch, n_q_heads, n_kv_heads, head_dim;
    int32_t q_len;      /* query rows per sequence (T for prefill, 1 for decode) */
    int32_t max_kv_len; /* T of a contiguous K/V, or max over kv_lens            */
    int32_t k, bq, bk;
    const int32_t *kv_lens;    /* [batch] or NULL => every sequence has max_kv_len */
    const int32_t *page_table; /* [batch, max_pages] or NULL => contiguous K/V      */
    int32_t page_size, max_pages;
    int32_t n_threads;         /* OpenMP threads for the batched calls (<=0: default) */
    int32_t n_sink, n_window;  /* sparse attention only: always-attended first keys / most recent keys */
    /* mask estimation only: sampling strides inside the block score (Sec. 3.2, last paragraph) and the
     * position of a branch's representative block (Sec. 3.1 uses the centre; the appendix ablates others) */
    int32_t b_sq, b_sk;        /* <= 1: every query row / every key of the block */
    int32_t rep_pos;           /* 0 centre, 1 first block, 2 last block of the branch */
    int32_t top_r;             /* 0 or >= head_dim: all channels; else channels kept per query row */
    /* Token bank with a vector-map page table (Sec. 3.3, "KV Token Index Translation"): a page-table entry
     * e >= 0 names page e of the pool passed as K / V (the GPU-resident bank), an entry e < 0 a miss, whose
     * page is read from page -e-1 of the backing pool (same layout).  touched [batch, max_pages] bytes (may be
     * NULL) receives 1 for every logical page of which a call reads a key row (other bytes are left alone). */
    const float *k_backing, *v_backing;
    uint8_t *touched;
    /* Ensemble sample (appendix "Ensemble Hierarchical Top-k Approximation"): sample 0 is the plain mask; a
     * sample e > 0 has a pseudo-random term of size ens_r added to the branch scores of its middle round. */
    int32_t ens_sample;
    uint32_t ens_seed;
    float ens_r;
} oracle_problem;

/* Statistics of one mask-estimation unit, used by the structural pins. */
typedef struct {
    int32_t rounds;           /* rounds in which at least one node was split      */
    int32_t first_chunk_max;  /* largest initial chunk, in key blocks             */
    int64_t reps_scored;      /* representative key blocks scored over all rounds */
} oracle_mask_stats;

/* One (sequence, kv head) key or value matrix, contiguous or paged. */
typedef struct {
    const float *base;      /* contiguous: row 0 of the sequence; paged: pool + kv_head*page_size*d */
    const int32_t *pages;   /* NULL, or this sequence's row of the page table                       */
    int32_t page_size;
    int64_t page_stride;    /* floats between two pool pages: n_kv_heads*page_size*d               */
    int32_t d;
    const float *backing;   /* like base, in the backing pool (pages of negative table entries)      */
    uint8_t *touched;       /* NULL, or this sequence's row of the map of pages read                 */
} kv_view;

static const float *kv_row(const kv_view *v, int64_t t)
{
    if (!v->pages) return v->base + t * v->d;
    int64_t page = v->pages[t / v->page_size];
    if (v->touched) v->touched[t / v->page_size] = 1;
    const float *pool = v->base;
    if (page < 0) { pool = v->backing; page = -page - 1; } /* a miss: the page lives in the backing pool */
    return pool + page * v->page_stride + (t % v->page_size) * (int64_t)v->d;
}

/* round(a/b) to the nearest integer, halves up, exact in integers
 * (the rounding operator of Sec. 3.1's chunk bounds). */
static int64_t rnd_div(int64_t a, int64_t b) { return (2 * a + b) / (2 * b); }

/* ------------------------------------------------------------------------ */
/* randomness of an ensemble sample                                          */
/* ------------------------------------------------------------------------ */

/* The paper's ensemble draws several masks "by adding randomness r_e to the branch direction" of a middle
 * iteration and says no more.  Reading taken here: in round floor(R/2) of the R = ceil(log2(ceil(Tb/kb)))
 * rounds of a query block (rounds counted from 0), the score that the top-k selection compares is
 * score + r_e * u with u uniform on [-1, 1); the other rounds, and sample 0, are untouched.  So that a GPU
 * implementation can draw the SAME u without exchanging random numbers, u is a counter-based value: the
 * 32-bit finalizer of MurmurHash3 absorbs seed, sample, sequence, head, query block and the representative
 * key block of the branch one after the other, and the top 24 bits of the result, read as an integer n,
 * give u = (n - 2^23) / 2^23 (exact in single precision).  The perturbed score is formed in single
 * precision, product first, then sum (each rounded once), which is the precision the decision is taken in. */
static uint32_t ens_fmix32(uint32_t x)
{
    x ^= x >> 16; x *= 0x85ebca6bu; x ^= x >> 13; x *= 0xc2b2ae35u; x ^= x >> 16;
    return x;
}

static float ens_uniform(uint32_t seed, int32_t sample, int32_t b, int32_t h, int32_t qb, int64_t rep_block)
{
    uint32_t x = ens_fmix32(seed ^ 0x9e3779b9u);
    x = ens_fmix32(x ^ (uint32_t)sample);
    x = ens_fmix32(x ^ (uint32_t)b);
    x = ens_fmix32(x ^ (uint32_t)h);
    x = ens_fmix32(x ^ (uint32_t)qb);
    x = ens_fmix32(x ^ (uint32_t)rep_block);
    return (float)((int32_t)(x >> 8) - (1 << 23)) / 8388608.0f;
}

typedef struct { int32_t sample; uint32_t seed; float r; int32_t b, h, qb; } ens_ctx;

/* ------------------------------------------------------------------------ */
/* mask estimation for one (sequence, query head, query block)  -- Alg. 1    */
/* ------------------------------------------------------------------------ */

/*
 * q        n_rows x d rows of the query block (n_rows <= bq; the last block may be short)
 * pos0     absolute position of the block's first row
 * K        keys of the sequence for this head's KV head
 * out      kb entries: first token position of every selected key block, ascending,
 *          then ORACLE_SENTINEL padding
 */
static void mask_unit(const float *q, int n_rows, int64_t pos0, const kv_view *K, int64_t kv_len,
                      int kb, int bk, int b_sq, int b_sk, int rep_pos, int top_r, const ens_ctx *ens,
                      int32_t *out, oracle_mask_stats *st)
{
    if (b_sq < 1) b_sq = 1;
    if (b_sk < 1) b_sk = 1;
    const int d = K->d;
    for (int j = 0; j < kb; ++j) out[j] = ORACLE_SENTINEL;
    if (st) { st->rounds = 0; st->first_chunk_max = 0; st->reps_scored = 0; }

    /* Visible prefix of this query block: keys up to its last row, capped by the length. */
    int64_t pos_last = pos0 + n_rows - 1;
    int64_t L = pos_last + 1 < kv_len ? pos_last + 1 : kv_len;
    if (L <= 0) return;
    int64_t Tb = (L + bk - 1) / bk; /* visible key blocks */

    int64_t *ns = malloc(sizeof(int64_t) * (size_t)kb), *ne = malloc(sizeof(int64_t) * (size_t)kb);
    int64_t *bs = malloc(sizeof(int64_t) * 2 * (size_t)kb), *be = malloc(sizeof(int64_t) * 2 * (size_t)kb);
    double *sc = malloc(sizeof(double) * 2 * (size_t)kb);
    char *keep = malloc(2 * (size_t)kb);

    /* Top-r approximation (appendix "Top-r Approximation", its equation for q.k): a query row's dot
     * products run over the r channels where |q| is largest only.  use[m*d + c] marks them; the
     * channels are taken one by one, largest |q| first, the lower channel among equals. */
    char *use = NULL;
    if (top_r > 0 && top_r < d) {
        use = calloc((size_t)n_rows * (size_t)d, 1);
        for (int m = 0; m < n_rows; ++m) {
            const float *qrow = q + (int64_t)m * d;
            for (int l = 0; l < top_r; ++l) {
                int arg = -1;
                for (int c = 0; c < d; ++c)
                    if (!use[(size_t)m * d + c] && (arg < 0 || fabs((double)qrow[c]) > fabs((double)qrow[arg]))) arg = c;
                use[(size_t)m * d + arg] = 1;
            }
        }
    }

    /* Initial nodes: kb equal chunks of the block range with rounded bounds
     * (Alg. 1 "set k nodes' initial start and end indices", block-wise per Sec. 3.2). */
    int n = 0;
    for (int j = 0; j < kb; ++j) {
        int64_t s = rnd_div((int64_t)j * Tb, kb), e = rnd_div((int64_t)(j + 1) * Tb, kb);
        if (e > s) {
            ns[n] = s; ne[n] = e; ++n;
            if (st && e - s > st->first_chunk_max) st->first_chunk_max = (int32_t)(e - s);
        }
    }

    /* rounds a block of this length runs, whatever its data: the longest initial node halves (rounding up)
     * until it is one block long */
    int n_rounds = 0;
    for (int64_t len = (Tb + kb - 1) / kb; len > 1; len = (len + 1) / 2) ++n_rounds;

    for (int round = 0;; ++round) {
        int any_split = 0;
        for (int j = 0; j < n; ++j) any_split |= (ne[j] - ns[j] > 1);
        if (!any_split) break; /* every branch has length 1 */
        if (st) st->rounds++;

        /* Split every node at its rounded midpoint into a left and a right branch. */
        int nb = 0;
        for (int j = 0; j < n; ++j) {
            int64_t mid = ns[j] + (ne[j] - ns[j]) / 2;
            if (mid > ns[j]) { bs[nb] = ns[j]; be[nb] = mid; ++nb; }
            bs[nb] = mid; be[nb] = ne[j]; ++nb;
        }

        /* Score each branch by its centre key block: max over the block's query rows and
         * the block's keys of the causally admissible dot products (Sec. 3.2, Alg. 1). */
        for (int b = 0; b < nb; ++b) {
            int64_t r = rep_pos == 1 ? bs[b] : rep_pos == 2 ? be[b] - 1 : bs[b] + (be[b] - bs[b]) / 2;
            double best = -INFINITY;
            for (int kk = 0; kk < bk; kk += b_sk) {      /* every b_sk-th key of the block */
                int64_t t = r * bk + kk;
                if (t >= kv_len) continue;
                const float *krow = kv_row(K, t);
                for (int m = 0; m < n_rows; m += b_sq) { /* every b_sq-th row of the query block */
                    if (t > pos0 + m) continue;
                    const float *qrow = q + (int64_t)m * d;
                    double dot = 0.0;
                    for (int c = 0; c < d; ++c)
                        if (!use || use[(size_t)m * d + c]) dot += (double)qrow[c] * (double)krow[c];
                    if (dot > best) best = dot;
                }
            }
            if (ens && ens->sample > 0 && round == n_rounds / 2) {
                /* ensemble sample: this round's selection sees score + r_e * u, in single precision */
                volatile float pert = ens->r * ens_uniform(ens->seed, ens->sample, ens->b, ens->h, ens->qb, r);
                volatile float moved = (float)best + pert;
                best = (double)moved;
            }
            sc[b] = best;
            if (st) st->reps_scored++;
        }

        /* Keep the kb best branches; equal scores go to the lower position; order is kept (Eq. 4). */
        if (nb <= kb) {
            memset(keep, 1, (size_t)nb);
        } else {
            for (int i = 0; i < nb; ++i) {
                int rank = 0;
                for (int j = 0; j < nb; ++j)
                    if (sc[j] > sc[i] || (sc[j] == sc[i] && j < i)) ++rank;
                keep[i] = rank < kb;
            }
        }
        n = 0;
        for (int i = 0; i < nb; ++i)
            if (keep[i]) { ns[n] = bs[i]; ne[n] = be[i]; ++n; }
    }

    for (int j = 0; j < n; ++j) out[j] = (int32_t)(ns[j] * bk);
    free(ns); free(ne); free(bs); free(be); free(sc); free(keep); free(use);
}

/* ------------------------------------------------------------------------ */
/* top-k masked attention for one (sequence, query head, query block) Eq. 2-3 */
/* ------------------------------------------------------------------------ */

static int cmp_i64(const void *a, const void *b)
{
    int64_t x = *(const int64_t *)a, y = *(const int64_t *)b;
    return (x > y) - (x < y);
}

/*
 * Key set of a row at position pos (Eq. 2-3 with the mask given by the selected blocks), optionally
 * united with the first n_sink keys ("global sink") and the n_window most recent keys ("local
 * sliding window"), which the paper adds in its block-sparse attention kernel (appendix, "Block
 * Sparse Flash Attention").  Every key counts once.
 */
static void attn_unit(const float *q, int n_rows, int64_t pos0, const kv_view *K, const kv_view *V,
                      int64_t kv_len, const int32_t *idx, int kb, int bk, double sm_scale,
                      int64_t n_sink, int64_t n_window, double *o)
{
    const int d = K->d;
    for (int m = 0; m < n_rows; ++m) {
        const float *qrow = q + (int64_t)m * d;
        double *orow = o + (int64_t)m * d;
        const int64_t pos = pos0 + m;
        for (int c = 0; c < d; ++c) orow[c] = 0.0;
        if (pos < 0) continue;
        const int64_t vis = pos + 1 < kv_len ? pos + 1 : kv_len; /* keys [0, vis) are admissible */
        const int64_t ns = n_sink < vis ? n_sink : vis;
        const int64_t w0 = vis - n_window > 0 ? vis - n_window : 0;
        size_t cap = (size_t)kb * (size_t)bk + (size_t)(ns > 0 ? ns : 0) + (size_t)(vis - w0) + 1;
        int64_t *ts = malloc(sizeof(int64_t) * cap);
        double *s = malloc(sizeof(double) * cap);
        size_t nk = 0;
        for (int j = 0; j < kb; ++j) {
            if (idx[j] < 0 || (int64_t)idx[j] >= kv_len) continue; /* sentinel / no block */
            for (int kk = 0; kk < bk; ++kk) {
                int64_t t = (int64_t)idx[j] + kk;
                if (t < vis) ts[nk++] = t;
            }
        }
        for (int64_t t = 0; t < ns; ++t) ts[nk++] = t;
        if (n_window > 0) for (int64_t t = w0; t < vis; ++t) ts[nk++] = t;
        qsort(ts, nk, sizeof(int64_t), cmp_i64);
        size_t nu = 0;
        for (size_t i = 0; i < nk; ++i)
            if (nu == 0 || ts[i] != ts[nu - 1]) ts[nu++] = ts[i];
        if (nu == 0) { free(ts); free(s); continue; } /* no admissible key: the row's output is zero */
        double mx = -INFINITY;
        for (size_t i = 0; i < nu; ++i) {
            const float *krow = kv_row(K, ts[i]);
            double dot = 0.0;
            for (int c = 0; c < d; ++c) dot += (double)qrow[c] * (double)krow[c];
            s[i] = sm_scale * dot;
            if (s[i] > mx) mx = s[i];
        }
        double den = 0.0;
        for (size_t i = 0; i < nu; ++i) { s[i] = exp(s[i] - mx); den += s[i]; }
        for (size_t i = 0; i < nu; ++i) {
            const float *vrow = kv_row(V, ts[i]);
            double pr = s[i] / den;
            for (int c = 0; c < d; ++c) orow[c] += pr * (double)vrow[c];
        }
        free(ts); free(s);
    }
}

/* ------------------------------------------------------------------------ */
/* exported entry points                                                     */
/* ------------------------------------------------------------------------ */

static kv_view make_view(const oracle_problem *p, const float *X, const float *backing, int b, int hkv)
{
    kv_view v;
    v.d = p->head_dim;
    v.backing = NULL; v.touched = NULL;
    if (p->page_table) {
        if (backing) v.backing = backing + (int64_t)hkv * p->page_size * p->head_dim;
        if (p->touched) v.touched = p->touched + (int64_t)b * p->max_pages;
        v.pages = p->page_table + (int64_t)b * p->max_pages;
        v.page_size = p->page_size;
        v.page_stride = (int64_t)p->n_kv_heads * p->page_size * p->head_dim;
        v.base = X + (int64_t)hkv * p->page_size * p->head_dim;
    } else {
        v.pages = NULL; v.page_size = 0; v.page_stride = 0;
        v.base = X + ((int64_t)b * p->n_kv_heads + hkv) * (int64_t)p->max_kv_len * p->head_dim;
    }
    return v;
}

static int check(const oracle_problem *p)
{
    if (!p || p->batch < 0 || p->n_q_heads <= 0 || p->n_kv_heads <= 0 || p->head_dim <= 0) return -1;
    if (p->n_q_heads % p->n_kv_heads) return -1;
    if (p->k <= 0 || p->bk <= 0 || p->bq <= 0 || p->k % p->bk) return -1;
    if (p->q_len < 0 || p->max_kv_len < 0) return -1;
    if (p->page_table && (p->page_size <= 0 || p->page_size % p->bk || p->max_pages <= 0)) return -1;
    return 0;
}

int32_t oracle_n_query_blocks(const oracle_problem *p) { return (p->q_len + p->bq - 1) / p->bq; }

/*
 * Mask estimation for a list of units.  A unit is (b, h, qb) packed as three int32.
 * Q  [batch, n_q_heads, q_len, d] contiguous floats
 * K  [batch, n_kv_heads, max_kv_len, d] contiguous floats, or the page pool
 *    [n_pages, n_kv_heads, page_size, d] when p->page_table is set
 * out[u*kb .. u*kb+kb) receives unit u's indices; stats (may be NULL) one entry per unit.
 */
int oracle_hip_mask_estimate_units(const oracle_problem *p, const float *Q, const float *K,
                                   const int32_t *units, int64_t n_units, int32_t *out,
                                   oracle_mask_stats *stats)
{
    if (check(p) || !Q || !K || !out || (n_units > 0 && !units)) return -1;
    const int kb = p->k / p->bk, d = p->head_dim, g = p->n_q_heads / p->n_kv_heads;
    int nthreads = p->n_threads;
    (void)nthreads;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads > 0 ? nthreads : 1)
#endif
    for (int64_t u = 0; u < n_units; ++u) {
        int b = units[3 * u], h = units[3 * u + 1], qb = units[3 * u + 2];
        int64_t kv_len = p->kv_lens ? p->kv_lens[b] : p->max_kv_len;
        int row0 = qb * p->bq;
        int n_rows = p->q_len - row0 < p->bq ? p->q_len - row0 : p->bq;
        int64_t pos0 = kv_len - p->q_len + row0;
        kv_view kv = make_view(p, K, p->k_backing, b, h / g);
        const float *q = Q + (((int64_t)b * p->n_q_heads + h) * p->q_len + row0) * d;
        ens_ctx ens = {p->ens_sample, p->ens_seed, p->ens_r, b, h, qb};
        mask_unit(q, n_rows, pos0, &kv, kv_len, kb, p->bk, p->b_sq, p->b_sk, p->rep_pos, p->top_r, &ens, out + u * kb,
                  stats ? stats + u : NULL);
    }
    return 0;
}

/* Sparse attention for a list of units; idx[u*kb ..) are unit u's block indices;
 * O[u*bq*d ..) receives bq x d doubles (rows past q_len are left untouched). */
int oracle_hip_sparse_attn_units(const oracle_problem *p, const float *Q, const float *K, const float *V,
                                 const int32_t *units, int64_t n_units, const int32_t *idx,
                                 double sm_scale, double *O)
{
    if (check(p) || !Q || !K || !V || !idx || !O || (n_units > 0 && !units)) return -1;
    const int kb = p->k / p->bk, d = p->head_dim, g = p->n_q_heads / p->n_kv_heads;
    if (!(sm_scale > 0.0)) sm_scale = 1.0 / sqrt((double)d);
    int nthreads = p->n_threads;
    (void)nthreads;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads > 0 ? nthreads : 1)
#endif
    for (int64_t u = 0; u < n_units; ++u) {
        int b = units[3 * u], h = units[3 * u + 1], qb = units[3 * u + 2];
        int64_t kv_len = p->kv_lens ? p->kv_lens[b] : p->max_kv_len;
        int row0 = qb * p->bq;
        int n_rows = p->q_len - row0 < p->bq ? p->q_len - row0 : p->bq;
        int64_t pos0 = kv_len - p->q_len + row0;
        kv_view kk = make_view(p, K, p->k_backing, b, h / g), vv = make_view(p, V, p->v_backing, b, h / g);
        const float *q = Q + (((int64_t)b * p->n_q_heads + h) * p->q_len + row0) * d;
        attn_unit(q, n_rows, pos0, &kk, &vv, kv_len, idx + u * kb, kb, p->bk, sm_scale,
                  p->n_sink > 0 ? p->n_sink : 0, p->n_window > 0 ? p->n_window : 0,
                  O + u * (int64_t)p->bq * d);
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* ensemble vote (appendix "Ensemble Hierarchical Top-k Approximation")      */
/* ------------------------------------------------------------------------ */

static int cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/*
 * samples [n_e][n_units][kb]: n_e index sets per query block (entries < 0 or == ORACLE_SENTINEL: no block;
 * a set holds a position at most once).  A position's votes = the number of sets that hold it.  Kept: the
 * positions with votes >= theta_vote (theta_vote = 1: union, = n_e: intersection).  tau = 1: at most kb of
 * them, those with more votes first, the lower position among equal votes.  out [n_units][width], width =
 * kb if tau else n_e * kb: the kept positions ascending, then ORACLE_SENTINEL padding.
 */
int oracle_hip_vote(const int32_t *samples, int32_t n_e, int64_t n_units, int32_t kb, int32_t theta_vote,
                    int32_t tau, int32_t *out)
{
    if (!samples || !out || n_e <= 0 || kb <= 0 || n_units < 0 || theta_vote < 1) return -1;
    const int64_t width = tau ? kb : (int64_t)n_e * kb;
    const size_t cap = (size_t)n_e * (size_t)kb;
    int32_t *all = malloc(sizeof(int32_t) * cap), *pos = malloc(sizeof(int32_t) * cap), *votes = malloc(sizeof(int32_t) * cap);
    for (int64_t u = 0; u < n_units; ++u) {
        size_t n = 0;
        for (int e = 0; e < n_e; ++e)
            for (int j = 0; j < kb; ++j) {
                int32_t v = samples[((int64_t)e * n_units + u) * kb + j];
                if (v >= 0 && v != ORACLE_SENTINEL) all[n++] = v;
            }
        qsort(all, n, sizeof(int32_t), cmp_i32);
        size_t m = 0; /* distinct positions with enough votes */
        for (size_t i = 0; i < n;) {
            size_t j = i;
            while (j < n && all[j] == all[i]) ++j;
            if ((int64_t)(j - i) >= theta_vote) { pos[m] = all[i]; votes[m] = (int32_t)(j - i); ++m; }
            i = j;
        }
        int32_t *row = out + u * width;
        int64_t w = 0;
        for (size_t i = 0; i < m; ++i) {
            int take = 1;
            if (tau && m > (size_t)kb) {
                size_t rank = 0; /* positions that come before this one: more votes, or as many at a lower position */
                for (size_t j = 0; j < m; ++j)
                    if (votes[j] > votes[i] || (votes[j] == votes[i] && j < i)) ++rank;
                take = rank < (size_t)kb;
            }
            if (take) row[w++] = pos[i];
        }
        for (; w < width; ++w) row[w] = ORACLE_SENTINEL;
    }
    free(all); free(pos); free(votes);
    return 0;
}

static int32_t *all_units(const oracle_problem *p, int64_t *n_units)
{
    int nqb = oracle_n_query_blocks(p);
    *n_units = (int64_t)p->batch * p->n_q_heads * nqb;
    int32_t *u = malloc(sizeof(int32_t) * 3 * (size_t)(*n_units > 0 ? *n_units : 1));
    int64_t i = 0;
    for (int b = 0; b < p->batch; ++b)
        for (int h = 0; h < p->n_q_heads; ++h)
            for (int qb = 0; qb < nqb; ++qb) { u[3 * i] = b; u[3 * i + 1] = h; u[3 * i + 2] = qb; ++i; }
    return u;
}

/* Whole problem: indices [batch, n_q_heads, ceil(q_len/bq), k/bk]. */
int oracle_hip_mask_estimate(const oracle_problem *p, const float *Q, const float *K, int32_t *indices)
{
    if (check(p)) return -1;
    int64_t n;
    int32_t *u = all_units(p, &n);
    int rc = oracle_hip_mask_estimate_units(p, Q, K, u, n, indices, NULL);
    free(u);
    return rc;
}

/* Whole problem: O [batch, n_q_heads, q_len, d] doubles. */
int oracle_hip_sparse_attn(const oracle_problem *p, const float *Q, const float *K, const float *V,
                           const int32_t *indices, double sm_scale, double *O)
{
    if (check(p) || !O) return -1;
    int64_t n;
    int32_t *u = all_units(p, &n);
    const int d = p->head_dim, nqb = oracle_n_query_blocks(p);
    double *tmp = malloc(sizeof(double) * (size_t)(n > 0 ? n : 1) * (size_t)p->bq * (size_t)d);
    int rc = oracle_hip_sparse_attn_units(p, Q, K, V, u, n, indices, sm_scale, tmp);
    if (rc == 0) {
        for (int64_t i = 0; i < n; ++i) {
            int b = u[3 * i], h = u[3 * i + 1], qb = u[3 * i + 2];
            int row0 = qb * p->bq;
            int n_rows = p->q_len - row0 < p->bq ? p->q_len - row0 : p->bq;
            double *dst = O + (((int64_t)b * p->n_q_heads + h) * p->q_len + row0) * d;
            memcpy(dst, tmp + i * (int64_t)p->bq * d, sizeof(double) * (size_t)n_rows * (size_t)d);
        }
    }
    (void)nqb;
    free(tmp); free(u);
    return rc;
}
