// Host-side launchers of the kernel families (one translation unit each).
#pragma once
#include "common.h"

namespace hipattn {

hipError_t launch_mask_generic(const KParams &p, bool bf16, hipStream_t st);
bool mask_mfma_supported(const KParams &p, bool bf16);
hipError_t launch_mask_mfma(const KParams &p, hipStream_t st);
bool attn_mfma_supported(const KParams &p, bool bf16);
hipError_t launch_attn_mfma(const KParams &p, hipStream_t st);
hipError_t launch_attn_mfma_direct(const KParams &p, dim3 grid, int log_bk, int mtn, int xcd_map, int mode, bool split, hipStream_t st);
bool mask_decode_supported(const KParams &p, bool bf16);
hipError_t launch_mask_decode(const KParams &p, hipStream_t st);
bool attn_decode_supported(const KParams &p, bool bf16);
hipError_t launch_attn_decode(const KParams &p, hipStream_t st);
hipError_t launch_attn_generic(const KParams &p, bool bf16, hipStream_t st);
hipError_t launch_topr_mask(const KParams &p, bool bf16, void *dst, hipStream_t st);
hipError_t launch_touch_attn(const KParams &p, hipStream_t st);
bool vote_supported(int n_e, int kb);
hipError_t launch_vote(const int32_t *samples, int32_t *out, int64_t n_units, int n_e, int kb, int theta, int tau, hipStream_t st);

}  // namespace hipattn
