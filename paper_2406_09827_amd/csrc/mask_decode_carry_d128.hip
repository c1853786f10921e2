// Instantiates the decode mask-estimation kernels: scores carried from parent to child (first / last representative), head dim 128.
#include "mask_decode_impl.h"

namespace hipattn {
template hipError_t launch_mask_decode_variant<true, 128>(const KParams &, hipStream_t);
}  // namespace hipattn
