// Instantiates the prefill mask-estimation kernels for 1 scored key row per block (bk / b_sk).
#include "mask_mfma_impl.h"

namespace hipattn {
template hipError_t launch_mask_mfma_lb<0>(const KParams &, hipStream_t);
}  // namespace hipattn
