// Dispatch of the matrix-core prefill mask-estimation kernels (see mask_mfma_impl.h).
#include "common.h"
#include "launch.h"

namespace hipattn {

template <int LB> hipError_t launch_mask_mfma_lb(const KParams &p, hipStream_t st);
extern template hipError_t launch_mask_mfma_lb<0>(const KParams &, hipStream_t);
extern template hipError_t launch_mask_mfma_lb<1>(const KParams &, hipStream_t);
extern template hipError_t launch_mask_mfma_lb<2>(const KParams &, hipStream_t);
extern template hipError_t launch_mask_mfma_lb<3>(const KParams &, hipStream_t);

bool mask_mfma_supported(const KParams &p, bool bf16)
{
    // bf16 prefill with 1, 2, 4 (or, at head dim 128, 8) scored key rows per block (bk / b_sk) and k/bk <= 1024; everything else goes to
    // the generic kernel.  The contiguous variant addresses key rows by 32-bit byte offsets from
    // the start of a (sequence, kv head) slice, formed with a 24-bit multiply (row number x row pitch).
    // The paged variant adds a 32-bit offset inside the page to a 64-bit page base; page sizes that are
    // not a power of two go to the generic kernel.
    const bool fits32 = p.page_table ? (p.page_shift >= 0 && p.ks_b * 2 < (1LL << 32) && p.page_size < (1 << 24) && p.ks_r * 2 < (1 << 24) &&
                                        (int64_t)p.page_size * p.ks_r * 2 < (1LL << 31))
                                     : ((int64_t)p.max_kv_len * p.ks_r * 2 < (1LL << 31) && p.max_kv_len < (1 << 24) &&
                                        p.ks_r * 2 < (1 << 24));
    const auto pow2 = [](int v) { return v > 0 && (v & (v - 1)) == 0; };
    const int rows = p.bk / p.b_sk;  // key rows scored per block
    // 1024 branch slots with one query tile: list rounds pack (slot, block index) into one word, 21 bits of index
    const bool one_tile = (p.bq + p.b_sq - 1) / p.b_sq <= 32;
    if (p.kb > 256 && p.kb <= 512 && one_tile && (p.max_kv_len + p.bk - 1) / p.bk >= (1 << 21)) return false;
    return bf16 && p.q_len > 1 && pow2(p.bk) && pow2(p.b_sk) && pow2(p.b_sq) && (rows == 1 || rows == 2 || rows == 4 || (rows == 8 && p.d == 128)) &&
           p.bq <= 64 && p.kb <= 1024 && fits32;
}

hipError_t launch_mask_mfma(const KParams &p, hipStream_t st)
{
    const int rows = p.bk / p.b_sk;
    if (rows == 1) return launch_mask_mfma_lb<0>(p, st);
    if (rows == 2) return launch_mask_mfma_lb<1>(p, st);
    if (rows == 4) return launch_mask_mfma_lb<2>(p, st);
    return launch_mask_mfma_lb<3>(p, st);
}

}  // namespace hipattn
