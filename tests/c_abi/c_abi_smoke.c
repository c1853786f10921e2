/*
 * Plain C caller of the hipattn C ABI (no Python, no torch): allocates device buffers with the HIP
 * runtime, runs hip_mask_estimate and hip_sparse_attn on a small fp32 problem and checks two facts
 * that need no oracle:
 *   1. with k >= T every visible key block is selected: indices of query block qb are 0, bk, 2*bk, ...
 *      up to its visible prefix, then HIP_ATTN_SENTINEL;
 *   2. with V[t][c] = 1 for every t, c the attention output is 1 for every row (softmax weights sum to 1).
 * Exit code 0 = both hold.
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "hipattn.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 2; } } while (0)

int main(void)
{
    enum { B = 1, HQ = 2, HKV = 1, D = 64, T = 96, BQ = 16, BK = 2, K = 128 };  /* kb = 64 >= T/bk = 48 */
    const int nqb = T / BQ, kb = K / BK;
    const size_t nq = (size_t)B * HQ * T * D, nkv = (size_t)B * HKV * T * D, ni = (size_t)B * HQ * nqb * kb;
    float *hq = malloc(nq * sizeof(float)), *hk = malloc(nkv * sizeof(float)), *hv = malloc(nkv * sizeof(float));
    float *ho = malloc(nq * sizeof(float));
    int32_t *hi = malloc(ni * sizeof(int32_t));
    for (size_t i = 0; i < nq; ++i) hq[i] = (float)((int)(i * 7 % 9) - 4) / 8.0f;
    for (size_t i = 0; i < nkv; ++i) { hk[i] = (float)((int)(i * 5 % 9) - 4) / 8.0f; hv[i] = 1.0f; }

    float *dq, *dk, *dv, *dout;
    int32_t *di;
    CHECK_HIP(hipMalloc((void **)&dq, nq * sizeof(float)));
    CHECK_HIP(hipMalloc((void **)&dk, nkv * sizeof(float)));
    CHECK_HIP(hipMalloc((void **)&dv, nkv * sizeof(float)));
    CHECK_HIP(hipMalloc((void **)&dout, nq * sizeof(float)));
    CHECK_HIP(hipMalloc((void **)&di, ni * sizeof(int32_t)));
    CHECK_HIP(hipMemcpy(dq, hq, nq * sizeof(float), hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(dk, hk, nkv * sizeof(float), hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(dv, hv, nkv * sizeof(float), hipMemcpyHostToDevice));

    hip_problem p;
    memset(&p, 0, sizeof p);
    p.batch = B; p.n_q_heads = HQ; p.n_kv_heads = HKV; p.head_dim = D;
    p.q_len = T; p.max_kv_len = T; p.k = K; p.bq = BQ; p.bk = BK; p.dtype = HIP_ATTN_F32;

    int rc = hip_mask_estimate(&p, dq, dk, di, NULL);
    if (rc != HIP_ATTN_OK) { fprintf(stderr, "hip_mask_estimate: %s\n", hip_strerror(rc)); return 1; }
    rc = hip_sparse_attn(&p, dq, dk, dv, di, dout, NULL);
    if (rc != HIP_ATTN_OK) { fprintf(stderr, "hip_sparse_attn: %s\n", hip_strerror(rc)); return 1; }
    CHECK_HIP(hipDeviceSynchronize());
    CHECK_HIP(hipMemcpy(hi, di, ni * sizeof(int32_t), hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(ho, dout, nq * sizeof(float), hipMemcpyDeviceToHost));

    int bad = 0;
    for (int h = 0; h < HQ; ++h)
        for (int qb = 0; qb < nqb; ++qb) {
            const int visible = (qb + 1) * BQ / BK;  /* key blocks up to the block's last row */
            const int32_t *row = hi + ((size_t)h * nqb + qb) * kb;
            for (int j = 0; j < kb; ++j) {
                const int32_t want = j < visible ? j * BK : HIP_ATTN_SENTINEL;
                if (row[j] != want) { if (!bad) fprintf(stderr, "index h=%d qb=%d j=%d: %d, expected %d\n", h, qb, j, row[j], want); ++bad; }
            }
        }
    for (size_t i = 0; i < nq; ++i)
        if (fabsf(ho[i] - 1.0f) > 1e-5f) { if (!bad) fprintf(stderr, "output %zu: %g, expected 1\n", i, ho[i]); ++bad; }
    /* an argument error comes back as a code, before any launch */
    p.head_dim = 80;
    if (hip_mask_estimate(&p, dq, dk, di, NULL) != HIP_ATTN_EHEADDIM) { fprintf(stderr, "head_dim 80 not rejected\n"); ++bad; }
    printf("c_abi_smoke: version %d, %s\n", hip_attn_version(), bad ? "FAILED" : "ok");
    hipFree(dq); hipFree(dk); hipFree(dv); hipFree(dout); hipFree(di);
    free(hq); free(hk); free(hv); free(ho); free(hi);
    return bad ? 1 : 0;
}
