// Instantiates the prefill mask-estimation kernels for key blocks of 4 tokens.
#include "mask_mfma_impl.h"

namespace hipattn {
template hipError_t launch_mask_mfma_lb<2>(const KParams &, hipStream_t);
}  // namespace hipattn
