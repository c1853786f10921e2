// Decode mask estimation: dispatch over the variants (each instantiated in its own translation unit).
#include "mask_decode_impl.h"

namespace hipattn {

extern template hipError_t launch_mask_decode_variant<64, false>(const KParams &, hipStream_t);
extern template hipError_t launch_mask_decode_variant<64, true>(const KParams &, hipStream_t);
extern template hipError_t launch_mask_decode_variant<128, false>(const KParams &, hipStream_t);
extern template hipError_t launch_mask_decode_variant<128, true>(const KParams &, hipStream_t);

bool mask_decode_supported(const KParams &p, bool bf16)
{
    const int rows = p.bk / p.b_sk;  // key rows scored per block
    return bf16 && p.q_len == 1 && p.bq == 1 && (rows == 1 || rows == 2 || rows == 4 || rows == 8) && p.kb <= 1024;
}

hipError_t launch_mask_decode(const KParams &p, hipStream_t st)
{
    const bool wide = p.bk / p.b_sk >= 4;
    if (p.d == 64) return wide ? launch_mask_decode_variant<64, true>(p, st) : launch_mask_decode_variant<64, false>(p, st);
    return wide ? launch_mask_decode_variant<128, true>(p, st) : launch_mask_decode_variant<128, false>(p, st);
}

}  // namespace hipattn
