// Dispatch of the matrix-core prefill mask-estimation kernels (see mask_mfma_impl.h).
#include "common.h"
#include "launch.h"

namespace hipattn {

template <int LB> hipError_t launch_mask_mfma_lb(const KParams &p, hipStream_t st);
extern template hipError_t launch_mask_mfma_lb<0>(const KParams &, hipStream_t);
extern template hipError_t launch_mask_mfma_lb<1>(const KParams &, hipStream_t);
extern template hipError_t launch_mask_mfma_lb<2>(const KParams &, hipStream_t);

bool mask_mfma_supported(const KParams &p, bool bf16)
{
    // bf16 prefill with key blocks of 1, 2 or 4 tokens and k/bk <= 512; everything else goes to
    // the generic kernel.  The contiguous variant addresses key rows by 32-bit byte offsets from
    // the start of a (sequence, kv head) slice.
    const bool fits32 = p.page_table || (int64_t)p.max_kv_len * p.ks_r * 2 < (1LL << 31);
    return bf16 && p.q_len > 1 && (p.bk == 1 || p.bk == 2 || p.bk == 4) && p.bq <= 64 && p.kb <= 512 && fits32;
}

hipError_t launch_mask_mfma(const KParams &p, hipStream_t st)
{
    if (p.bk == 1) return launch_mask_mfma_lb<0>(p, st);
    if (p.bk == 2) return launch_mask_mfma_lb<1>(p, st);
    return launch_mask_mfma_lb<2>(p, st);
}

}  // namespace hipattn
