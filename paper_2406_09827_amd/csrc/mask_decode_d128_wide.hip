// Instantiates the decode mask-estimation kernels: head dim 128, 4 or 8 scored key rows per block.
#include "mask_decode_impl.h"

namespace hipattn {
template hipError_t launch_mask_decode_variant<128, true>(const KParams &, hipStream_t);
}  // namespace hipattn
