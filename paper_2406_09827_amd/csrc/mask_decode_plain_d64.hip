// Instantiates the decode mask-estimation kernels: centre representative, head dim 64.
#include "mask_decode_impl.h"

namespace hipattn {
template hipError_t launch_mask_decode_variant<false, 64>(const KParams &, hipStream_t);
}  // namespace hipattn
