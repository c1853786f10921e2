"""HiP (Hierarchically Pruned Attention) hot path for AMD MI355X.

`hip_mask_estimate` and `hip_sparse_attn` call the C-ABI library libhipattn.so
(hand-written HIP kernels for gfx950); see include/hipattn.h for the contract.
"""
from .binding import (BF16, F32, FORCE_GENERIC, SENTINEL, HipAttnError, HipProblem, hip_mask_estimate, hip_mask_estimate_noalloc, hip_mask_ensemble,
                      hip_mask_vote,                      hip_sparse_attn, load, make_problem)

__all__ = ["hip_mask_estimate", "hip_mask_estimate_noalloc", "hip_mask_vote", "hip_mask_ensemble", "hip_sparse_attn", "make_problem", "load", "HipProblem", "HipAttnError",
           "SENTINEL", "F32", "BF16", "FORCE_GENERIC"]
