// Decode mask estimation: the default variant (centre representative) and the dispatch.
#include "mask_decode_impl.h"

namespace hipattn {

hipError_t launch_mask_decode_carry(const KParams &p, hipStream_t st);  // mask_decode_carry.hip

bool mask_decode_supported(const KParams &p, bool bf16)
{
    const int rows = p.bk / p.b_sk;  // key rows scored per block
    return bf16 && p.q_len == 1 && p.bq == 1 && (rows == 1 || rows == 2 || rows == 4 || rows == 8) && p.kb <= 1024;
}

hipError_t launch_mask_decode(const KParams &p, hipStream_t st)
{
    return p.rep_pos != 0 ? launch_mask_decode_carry(p, st) : launch_mask_decode_variant<false>(p, st);
}

}  // namespace hipattn
