// Instantiates the prefill mask-estimation kernels for 2 scored key rows per block (bk / b_sk).
#include "mask_mfma_impl.h"

namespace hipattn {
template hipError_t launch_mask_mfma_lb<1>(const KParams &, hipStream_t);
}  // namespace hipattn
