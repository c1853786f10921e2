// Decode mask estimation: dispatch over the variants (each instantiated in its own translation unit).
#include "mask_decode_impl.h"

namespace hipattn {

extern template hipError_t launch_mask_decode_variant<false, 64>(const KParams &, hipStream_t);
extern template hipError_t launch_mask_decode_variant<false, 128>(const KParams &, hipStream_t);
extern template hipError_t launch_mask_decode_variant<true, 64>(const KParams &, hipStream_t);
extern template hipError_t launch_mask_decode_variant<true, 128>(const KParams &, hipStream_t);

bool mask_decode_supported(const KParams &p, bool bf16)
{
    const int rows = p.bk / p.b_sk;  // key rows scored per block
    return bf16 && p.q_len == 1 && p.bq == 1 && (rows == 1 || rows == 2 || rows == 4 || rows == 8) && p.kb <= 1024;
}

hipError_t launch_mask_decode(const KParams &p, hipStream_t st)
{
    // first / last representative: the variant that carries a node's score to the child sharing its representative
    if (p.rep_pos != 0) return p.d == 64 ? launch_mask_decode_variant<true, 64>(p, st) : launch_mask_decode_variant<true, 128>(p, st);
    return p.d == 64 ? launch_mask_decode_variant<false, 64>(p, st) : launch_mask_decode_variant<false, 128>(p, st);
}

}  // namespace hipattn
