// C ABI of the HiP attention library: argument validation and kernel dispatch.
#include "../../include/hipattn.h"
#include "common.h"
#include "launch.h"

#include <mutex>

using namespace hipattn;

// Scratch of hip_mask_estimate_noalloc: lives in the code object, one copy per GPU the library is loaded on,
// held until the process ends.  In host code this name is only a handle for hipGetSymbolAddress.
static __device__ __align__(256) unsigned char scratch[HIP_ATTN_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each GPU, looked up once per GPU
std::mutex g_scratch_mutex;

// Device address of this GPU's copy of `scratch` (nullptr + error code on failure).
void *static_scratch(hipError_t &err)
{
    int dev = -1;
    err = hipGetDevice(&dev);
    if (err != hipSuccess) return nullptr;
    if (dev < 0 || dev >= kMaxDevices) { err = hipErrorInvalidDevice; return nullptr; }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));  // with device `dev` current: its own copy
        if (err != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Validates the problem and fills the kernel-side view.  Returns HIP_ATTN_OK or an error.
int prepare(const hip_problem *hp, KParams &kp)
{
    if (!hp) return HIP_ATTN_ENULL;
    const hip_problem &p = *hp;
    if (p.batch < 0 || p.n_q_heads <= 0 || p.n_kv_heads <= 0 || p.q_len < 0 || p.max_kv_len < 0) return HIP_ATTN_ESHAPE;
    if (p.n_q_heads % p.n_kv_heads) return HIP_ATTN_ESHAPE;
    if (p.q_len > p.max_kv_len) return HIP_ATTN_ESHAPE;
    if (p.n_sink < 0 || p.n_window < 0 || p.top_r < 0) return HIP_ATTN_ESHAPE;
    if (p.head_dim != 64 && p.head_dim != 128) return HIP_ATTN_EHEADDIM;
    if (p.dtype != HIP_ATTN_F32 && p.dtype != HIP_ATTN_BF16) return HIP_ATTN_EDTYPE;
    if (p.k <= 0 || p.bk <= 0 || p.bq <= 0 || p.k % p.bk) return HIP_ATTN_EBLOCK;
    if (p.bq > HIP_ATTN_MAX_BQ || p.bk > HIP_ATTN_MAX_BK) return HIP_ATTN_EBLOCK;
    if (p.b_sq < 0 || p.b_sk < 0 || p.b_sq > p.bq || (p.b_sk > 1 && p.bk % p.b_sk)) return HIP_ATTN_EBLOCK;
    if (p.rep_pos < HIP_ATTN_REP_CENTER || p.rep_pos > HIP_ATTN_REP_LAST) return HIP_ATTN_EBLOCK;
    if (p.k / p.bk > HIP_ATTN_MAX_KB) return HIP_ATTN_ETOOLARGE;
    if (p.page_table && (p.page_size <= 0 || p.page_size % p.bk || p.max_pages <= 0)) return HIP_ATTN_EPAGE;
    if (p.page_table && (int64_t)p.max_pages * p.page_size < p.max_kv_len) return HIP_ATTN_EPAGE;
    if (!p.page_table && (p.k_backing || p.v_backing || p.touched)) return HIP_ATTN_EPAGE;

    const int d = p.head_dim;
    const int nqb = (p.q_len + p.bq - 1) / p.bq;
    if ((int64_t)p.batch * p.n_q_heads * nqb > 0x7fffffffLL) return HIP_ATTN_ETOOLARGE;
    kp = KParams{};
    kp.batch = p.batch; kp.hq = p.n_q_heads; kp.hkv = p.n_kv_heads; kp.g = p.n_q_heads / p.n_kv_heads;
    kp.d = d; kp.q_len = p.q_len; kp.max_kv_len = p.max_kv_len;
    kp.kb = p.k / p.bk; kp.bq = p.bq; kp.bk = p.bk; kp.nqb = nqb;
    // a single query row is a one-row query block whatever bq says: the decode kernels then serve it
    if (p.q_len == 1) kp.bq = 1;
    kp.kv_lens = p.kv_lens; kp.page_table = p.page_table;
    kp.Kback = p.k_backing; kp.Vback = p.v_backing; kp.touched = p.touched;
    kp.page_size = p.page_size; kp.max_pages = p.max_pages;
    kp.n_sink = p.n_sink; kp.n_window = p.n_window;
    kp.b_sq = (p.b_sq > 1 && p.q_len > 1) ? p.b_sq : 1; kp.b_sk = p.b_sk > 1 ? p.b_sk : 1; kp.rep_pos = p.rep_pos;
    kp.top_r = p.top_r >= p.head_dim ? 0 : p.top_r;
    kp.flags = p.flags;
    kp.ens_sample = p.ens_sample > 0 ? p.ens_sample : 0; kp.ens_seed = p.ens_seed; kp.ens_r = p.ens_r;
    kp.page_shift = -1;
    if (p.page_table && (p.page_size & (p.page_size - 1)) == 0)
        for (kp.page_shift = 0; (1 << kp.page_shift) < p.page_size;) ++kp.page_shift;
    kp.sm_scale = p.sm_scale > 0.f ? p.sm_scale : 1.0f / sqrtf((float)d);

    auto all_zero = [](const int64_t s[3]) { return s[0] == 0 && s[1] == 0 && s[2] == 0; };
    if (all_zero(p.q_strides)) { kp.qs_r = d; kp.qs_h = (int64_t)p.q_len * d; kp.qs_b = kp.qs_h * p.n_q_heads; }
    else { kp.qs_b = p.q_strides[0]; kp.qs_h = p.q_strides[1]; kp.qs_r = p.q_strides[2]; }
    if (all_zero(p.o_strides)) { kp.os_r = d; kp.os_h = (int64_t)p.q_len * d; kp.os_b = kp.os_h * p.n_q_heads; }
    else { kp.os_b = p.o_strides[0]; kp.os_h = p.o_strides[1]; kp.os_r = p.o_strides[2]; }
    if (all_zero(p.kv_strides)) {
        const int64_t rows = p.page_table ? p.page_size : p.max_kv_len;
        kp.ks_r = d; kp.ks_h = rows * d; kp.ks_b = kp.ks_h * p.n_kv_heads;
    } else { kp.ks_b = p.kv_strides[0]; kp.ks_h = p.kv_strides[1]; kp.ks_r = p.kv_strides[2]; }

    // rows must stay 16-byte aligned for the 128-bit loads of the tuned kernels
    const int64_t per16 = p.dtype == HIP_ATTN_BF16 ? 8 : 4;
    const int64_t strides[] = {kp.qs_b, kp.qs_h, kp.qs_r, kp.ks_b, kp.ks_h, kp.ks_r, kp.os_b, kp.os_h, kp.os_r};
    for (int64_t s : strides)
        if (s < 0 || s % per16) return HIP_ATTN_EALIGN;
    if (kp.qs_r < d || kp.ks_r < d || kp.os_r < d) return HIP_ATTN_ESHAPE;
    return HIP_ATTN_OK;
}

int launch_result(hipError_t e) { return e == hipSuccess ? HIP_ATTN_OK : HIP_ATTN_ELAUNCH - (int)e; }

}  // namespace

extern "C" {

// Both mask-estimation entry points: `own_scratch` = use the library's static scratch instead of p->workspace.
static int mask_estimate_impl(const hip_problem *p, const void *Q, const void *K, int32_t *indices, void *stream,
                              bool own_scratch)
{
    KParams kp;
    int rc = prepare(p, kp);
    if (rc != HIP_ATTN_OK) return rc;
    if (kp.batch == 0 || kp.q_len == 0) return HIP_ATTN_OK;  // no work units: nothing is read or written
    if (!Q || !K || !indices) return HIP_ATTN_ENULL;
    if (!aligned16(Q) || !aligned16(K)) return HIP_ATTN_EALIGN;
    if (p->k_backing && !aligned16(p->k_backing)) return HIP_ATTN_EALIGN;
    kp.Q = Q; kp.K = K; kp.idx_out = indices;
    if (!kp.Kback) kp.Kback = K;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool bf16 = p->dtype == HIP_ATTN_BF16;
    const bool generic = p->flags & HIP_ATTN_FORCE_GENERIC;
    if (kp.top_r > 0) {
        // top-r scores: a copy of Q with the unused channels of every row zeroed goes to the scratch,
        // and the kernels below read that copy (dense layout)
        void *ws = p->workspace;
        if (own_scratch) {
            if (hip_workspace_bytes(p) > HIP_ATTN_STATIC_SCRATCH_BYTES) return HIP_ATTN_ESCRATCH;
            hipError_t e;
            ws = static_scratch(e);
            if (!ws) return launch_result(e);
        } else {
            if (!ws) return HIP_ATTN_ENULL;
            if (!aligned16(ws)) return HIP_ATTN_EALIGN;
            if (p->workspace_bytes < hip_workspace_bytes(p)) return HIP_ATTN_EWORKSPACE;
        }
        hipError_t e = launch_topr_mask(kp, bf16, ws, st);
        if (e != hipSuccess) return launch_result(e);
        kp.Q = ws;
        kp.qs_r = kp.d; kp.qs_h = (int64_t)kp.q_len * kp.d; kp.qs_b = kp.qs_h * kp.hq;
        kp.top_r = 0;
    }
    if (!generic && mask_mfma_supported(kp, bf16)) return launch_result(launch_mask_mfma(kp, st));
    if (!generic && mask_decode_supported(kp, bf16)) return launch_result(launch_mask_decode(kp, st));
    return launch_result(launch_mask_generic(kp, bf16, st));
}

int hip_mask_estimate(const hip_problem *p, const void *Q, const void *K, int32_t *indices, void *stream)
{
    return mask_estimate_impl(p, Q, K, indices, stream, false);
}

int hip_mask_vote(const hip_problem *p, const int32_t *samples, int32_t n_e, int32_t theta_vote, int32_t tau,
                  int32_t *indices, void *stream)
{
    KParams kp;
    int rc = prepare(p, kp);
    if (rc != HIP_ATTN_OK) return rc;
    if (!vote_supported(n_e, kp.kb) || theta_vote < 1) return HIP_ATTN_EENSEMBLE;
    if (kp.batch == 0 || kp.q_len == 0) return HIP_ATTN_OK;
    if (!samples || !indices) return HIP_ATTN_ENULL;
    const int64_t n_units = (int64_t)kp.batch * kp.hq * kp.nqb;
    return launch_result(launch_vote(samples, indices, n_units, n_e, kp.kb, theta_vote, tau ? 1 : 0,
                                     static_cast<hipStream_t>(stream)));
}

static size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

size_t hip_ensemble_workspace_bytes(const hip_problem *p, int32_t n_e)
{
    if (!p || n_e <= 0 || p->batch <= 0 || p->n_q_heads <= 0 || p->q_len <= 0 || p->bq <= 0 || p->bk <= 0 || p->k <= 0) return 0;
    const size_t nqb = (size_t)((p->q_len + p->bq - 1) / p->bq);
    const size_t one = (size_t)p->batch * (size_t)p->n_q_heads * nqb * (size_t)(p->k / p->bk) * sizeof(int32_t);
    return align256(hip_workspace_bytes(p)) + (size_t)n_e * one;
}

int hip_mask_ensemble(const hip_problem *p, const void *Q, const void *K, int32_t n_e, int32_t theta_vote,
                      int32_t tau, int32_t *indices, void *stream)
{
    KParams kp;
    int rc = prepare(p, kp);
    if (rc != HIP_ATTN_OK) return rc;
    if (!vote_supported(n_e, kp.kb) || theta_vote < 1) return HIP_ATTN_EENSEMBLE;
    if (kp.batch == 0 || kp.q_len == 0) return HIP_ATTN_OK;
    if (!p->workspace || !indices) return HIP_ATTN_ENULL;
    if (reinterpret_cast<uintptr_t>(p->workspace) & 255u) return HIP_ATTN_EALIGN;
    if (p->workspace_bytes < hip_ensemble_workspace_bytes(p, n_e)) return HIP_ATTN_EWORKSPACE;
    const size_t front = align256(hip_workspace_bytes(p));
    const size_t one = (hip_ensemble_workspace_bytes(p, n_e) - front) / (size_t)n_e;
    int32_t *samples = reinterpret_cast<int32_t *>(static_cast<char *>(p->workspace) + front);
    hip_problem q = *p;
    q.workspace_bytes = front;   // what is left to the top_r option
    for (int e = 0; e < n_e; ++e) {
        q.ens_sample = e;
        rc = mask_estimate_impl(&q, Q, K, samples + (size_t)e * (one / sizeof(int32_t)), stream, false);
        if (rc != HIP_ATTN_OK) return rc;
    }
    return hip_mask_vote(p, samples, n_e, theta_vote, tau, indices, stream);
}

int hip_mask_estimate_noalloc(const hip_problem *p, const void *Q, const void *K, int32_t *indices, void *stream)
{
    return mask_estimate_impl(p, Q, K, indices, stream, true);
}

int hip_sparse_attn(const hip_problem *p, const void *Q, const void *K, const void *V, const int32_t *indices,
                    void *O, void *stream)
{
    KParams kp;
    int rc = prepare(p, kp);
    if (rc != HIP_ATTN_OK) return rc;
    if (kp.batch == 0 || kp.q_len == 0) return HIP_ATTN_OK;
    if (!Q || !K || !V || !indices || !O) return HIP_ATTN_ENULL;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O)) return HIP_ATTN_EALIGN;
    kp.Q = Q; kp.K = K; kp.V = V; kp.O = O; kp.idx_in = indices;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool bf16 = p->dtype == HIP_ATTN_BF16;
    const bool generic = p->flags & HIP_ATTN_FORCE_GENERIC;
    if (p->k_backing && !aligned16(p->k_backing)) return HIP_ATTN_EALIGN;
    if (p->v_backing && !aligned16(p->v_backing)) return HIP_ATTN_EALIGN;
    if (!kp.Kback) kp.Kback = K;
    if (!kp.Vback) kp.Vback = V;
    hipError_t e;
    if (!generic && attn_mfma_supported(kp, bf16)) e = launch_attn_mfma(kp, st);
    else if (!generic && attn_decode_supported(kp, bf16)) e = launch_attn_decode(kp, st);
    else e = launch_attn_generic(kp, bf16, st);
    if (e == hipSuccess && kp.touched) e = launch_touch_attn(kp, st);  // the map of pages read, from the index array
    return launch_result(e);
}

size_t hip_workspace_bytes(const hip_problem *p)
{
    if (!p || p->top_r <= 0 || p->top_r >= p->head_dim) return 0;
    if (p->batch <= 0 || p->n_q_heads <= 0 || p->q_len <= 0 || p->head_dim <= 0) return 0;
    const size_t elem = p->dtype == HIP_ATTN_BF16 ? 2 : 4;
    return (size_t)p->batch * (size_t)p->n_q_heads * (size_t)p->q_len * (size_t)p->head_dim * elem;
}

const char *hip_strerror(int code)
{
    switch (code) {
        case HIP_ATTN_OK: return "ok";
        case HIP_ATTN_ENULL: return "a required pointer is NULL";
        case HIP_ATTN_ESHAPE: return "invalid shape (sizes, head grouping, q_len > kv_len or row stride < head_dim)";
        case HIP_ATTN_EBLOCK: return "invalid k / bq / bk or scoring options (k % bk != 0, block size out of range, sampling stride, representative)";
        case HIP_ATTN_EHEADDIM: return "head_dim must be 64 or 128";
        case HIP_ATTN_EDTYPE: return "dtype must be HIP_ATTN_F32 or HIP_ATTN_BF16";
        case HIP_ATTN_ETOOLARGE: return "k/bk or the number of work units exceeds the compiled maximum";
        case HIP_ATTN_EALIGN: return "pointer or stride not 16-byte aligned";
        case HIP_ATTN_EPAGE: return "invalid page table description (or a backing pool / touched map without a page table)";
        case HIP_ATTN_EWORKSPACE: return "workspace smaller than hip_workspace_bytes()";
        case HIP_ATTN_EENSEMBLE: return "ensemble: n_e outside 1..16, theta_vote < 1, or n_e * k/bk above 4096";
        case HIP_ATTN_ESCRATCH: return "the problem needs more scratch than the library's static HIP_ATTN_STATIC_SCRATCH_BYTES";
        default: return code <= HIP_ATTN_ELAUNCH ? "kernel launch failed" : "unknown error";
    }
}

int hip_attn_version(void) { return 106; }

}  // extern "C"
