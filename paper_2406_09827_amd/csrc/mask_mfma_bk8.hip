// Instantiates the prefill mask-estimation kernels for 8 scored key rows per block (bk / b_sk), head dim 128.
#include "mask_mfma_impl.h"

namespace hipattn {
template hipError_t launch_mask_mfma_lb<3>(const KParams &, hipStream_t);
}  // namespace hipattn
