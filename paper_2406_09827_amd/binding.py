"""Thin ctypes binding of libhipattn.so: argument marshalling only.

Every step of the method runs in the library's HIP kernels; torch tensors are used for
device memory and the current stream.  There is no CPU or eager fallback: if the shared
library is missing or a tensor is not on a GPU the call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhipattn.so")
SENTINEL = 2**31 - 1
F32, BF16 = 0, 1
FORCE_GENERIC = 1
NO_SHARED_ROUND = 2

EXPORTS = ("hip_mask_estimate", "hip_mask_estimate_noalloc", "hip_mask_vote", "hip_mask_ensemble",
           "hip_ensemble_workspace_bytes", "hip_sparse_attn", "hip_workspace_bytes", "hip_strerror", "hip_attn_version")


class HipProblem(ctypes.Structure):
    """Mirror of `hip_problem` in include/hipattn.h."""
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("q_len", ctypes.c_int32), ("max_kv_len", ctypes.c_int32),
        ("k", ctypes.c_int32), ("bq", ctypes.c_int32), ("bk", ctypes.c_int32),
        ("dtype", ctypes.c_int32), ("flags", ctypes.c_int32), ("sm_scale", ctypes.c_float),
        ("kv_lens", ctypes.c_void_p), ("page_table", ctypes.c_void_p),
        ("page_size", ctypes.c_int32), ("max_pages", ctypes.c_int32),
        ("q_strides", ctypes.c_int64 * 3), ("kv_strides", ctypes.c_int64 * 3), ("o_strides", ctypes.c_int64 * 3),
        ("n_sink", ctypes.c_int32), ("n_window", ctypes.c_int32),
        ("b_sq", ctypes.c_int32), ("b_sk", ctypes.c_int32), ("rep_pos", ctypes.c_int32), ("top_r", ctypes.c_int32),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
        ("k_backing", ctypes.c_void_p), ("v_backing", ctypes.c_void_p), ("touched", ctypes.c_void_p),
        ("ens_sample", ctypes.c_int32), ("ens_seed", ctypes.c_uint32), ("ens_r", ctypes.c_float),
    ]


_lib = None


def load() -> ctypes.CDLL:
    """Load the built library (build it first with `python -m paper_2406_09827_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built; run __graft_entry__.build() "
                               "(there is no fallback path)")
        lib = ctypes.CDLL(LIB_PATH)
        lib.hip_mask_estimate.restype = ctypes.c_int
        lib.hip_mask_estimate.argtypes = [ctypes.POINTER(HipProblem), ctypes.c_void_p, ctypes.c_void_p,
                                          ctypes.c_void_p, ctypes.c_void_p]
        lib.hip_mask_estimate_noalloc.restype = ctypes.c_int
        lib.hip_mask_estimate_noalloc.argtypes = lib.hip_mask_estimate.argtypes
        lib.hip_mask_vote.restype = ctypes.c_int
        lib.hip_mask_vote.argtypes = [ctypes.POINTER(HipProblem), ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32,
                                      ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p]
        lib.hip_mask_ensemble.restype = ctypes.c_int
        lib.hip_mask_ensemble.argtypes = [ctypes.POINTER(HipProblem), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32,
                                          ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p]
        lib.hip_ensemble_workspace_bytes.restype = ctypes.c_size_t
        lib.hip_ensemble_workspace_bytes.argtypes = [ctypes.POINTER(HipProblem), ctypes.c_int32]
        lib.hip_sparse_attn.restype = ctypes.c_int
        lib.hip_sparse_attn.argtypes = [ctypes.POINTER(HipProblem), ctypes.c_void_p, ctypes.c_void_p,
                                        ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        lib.hip_workspace_bytes.restype = ctypes.c_size_t
        lib.hip_workspace_bytes.argtypes = [ctypes.POINTER(HipProblem)]
        lib.hip_strerror.restype = ctypes.c_char_p
        lib.hip_strerror.argtypes = [ctypes.c_int]
        lib.hip_attn_version.restype = ctypes.c_int
        _lib = lib
    return _lib


class HipAttnError(RuntimeError):
    def __init__(self, code: int):
        self.code = code
        super().__init__(f"hipattn error {code}: {load().hip_strerror(code).decode()}")


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _need_gpu(*ts):
    for t in ts:
        if t is not None and not t.is_cuda:
            raise RuntimeError("hipattn needs device tensors (no CPU path exists)")


def make_problem(Q: torch.Tensor, K: torch.Tensor, k: int, bq: int, bk: int,
                 kv_lens: Optional[torch.Tensor] = None, page_table: Optional[torch.Tensor] = None,
                 max_kv_len: Optional[int] = None, sm_scale: float = 0.0, flags: int = 0,
                 O: Optional[torch.Tensor] = None) -> HipProblem:
    """Describe a call from tensor shapes/strides.  Q [B,Hq,Tq,d]; K [B,Hkv,T,d] or, with a
    page table, the pool [n_pages,Hkv,page,d]."""
    assert Q.dim() == 4 and K.dim() == 4 and Q.stride(3) == 1 and K.stride(3) == 1
    p = HipProblem()
    p.batch, p.n_q_heads, p.q_len, p.head_dim = Q.shape
    p.n_kv_heads = K.shape[1]
    if page_table is not None:
        assert page_table.dtype == torch.int32 and page_table.is_contiguous() and page_table.dim() == 2
        p.page_table = page_table.data_ptr()
        p.page_size = K.shape[2]
        p.max_pages = page_table.shape[1]
        p.max_kv_len = int(max_kv_len) if max_kv_len is not None else p.max_pages * p.page_size
    else:
        p.max_kv_len = K.shape[2] if max_kv_len is None else int(max_kv_len)
    if kv_lens is not None:
        assert kv_lens.dtype == torch.int32 and kv_lens.is_contiguous() and kv_lens.shape == (p.batch,)
        p.kv_lens = kv_lens.data_ptr()
    p.k, p.bq, p.bk = k, bq, bk
    p.dtype = _dtype_code(Q)
    p.flags = flags
    p.sm_scale = sm_scale
    p.q_strides = (ctypes.c_int64 * 3)(*Q.stride()[:3])
    p.kv_strides = (ctypes.c_int64 * 3)(*K.stride()[:3])
    if O is not None:
        p.o_strides = (ctypes.c_int64 * 3)(*O.stride()[:3])
    return p


def _token_bank(p: HipProblem, K, page_table, k_backing, v_backing, touched) -> None:
    """Backing pools for negative page-table entries and the map of pages read (see include/hipattn.h)."""
    for name, x in (("k_backing", k_backing), ("v_backing", v_backing)):
        if x is not None:
            # device memory or pinned host memory; same layout, strides and dtype as the bank
            assert page_table is not None and x.dim() == 4 and x.shape[1:] == K.shape[1:] and x.stride() == K.stride()
            assert x.dtype == K.dtype and (x.is_cuda or x.is_pinned())
            setattr(p, name, x.data_ptr())
    if touched is not None:
        assert page_table is not None and touched.is_cuda and touched.dtype == torch.uint8
        assert touched.is_contiguous() and touched.shape == page_table.shape
        p.touched = touched.data_ptr()


def _stream(t: torch.Tensor) -> int:
    return torch.cuda.current_stream(t.device).cuda_stream


def hip_mask_estimate(Q, K, k: int, bq: int, bk: int, kv_lens=None, page_table=None, max_kv_len=None,
                      flags: int = 0, indices: Optional[torch.Tensor] = None, b_sq: int = 1, b_sk: int = 1,
                      rep_pos: int = 0, top_r: int = 0, workspace: Optional[torch.Tensor] = None,
                      k_backing: Optional[torch.Tensor] = None, touched: Optional[torch.Tensor] = None,
                      ens_sample: int = 0, ens_seed: int = 0, ens_r: float = 0.0) -> torch.Tensor:
    """int32 indices [B, Hq, ceil(Tq/bq), k/bk] of the selected key blocks (see include/hipattn.h)."""
    _need_gpu(Q, K, kv_lens, page_table, indices)
    lib = load()
    p = make_problem(Q, K, k, bq, bk, kv_lens, page_table, max_kv_len, flags=flags)
    p.b_sq, p.b_sk, p.rep_pos, p.top_r = b_sq, b_sk, rep_pos, top_r
    p.ens_sample, p.ens_seed, p.ens_r = ens_sample, ens_seed & 0xffffffff, ens_r
    _token_bank(p, K, page_table, k_backing, None, touched)
    need = lib.hip_workspace_bytes(ctypes.byref(p))
    if need:
        if workspace is None:
            workspace = torch.empty(need, dtype=torch.uint8, device=Q.device)
        assert workspace.is_cuda and workspace.is_contiguous() and workspace.numel() * workspace.element_size() >= need
        p.workspace, p.workspace_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    nqb = (p.q_len + bq - 1) // bq
    if indices is None:
        indices = torch.empty((p.batch, p.n_q_heads, nqb, k // bk), dtype=torch.int32, device=Q.device)
    assert indices.dtype == torch.int32 and indices.is_contiguous()
    assert indices.numel() == p.batch * p.n_q_heads * nqb * (k // bk)
    rc = lib.hip_mask_estimate(ctypes.byref(p), Q.data_ptr(), K.data_ptr(), indices.data_ptr(), _stream(Q))
    if rc != 0:
        raise HipAttnError(rc)
    return indices


def hip_mask_vote(samples: torch.Tensor, theta_vote: int, tau: int, bq: int, bk: int, q_len: int,
                  indices: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Vote over samples [n_e, B, Hq, ceil(q_len/bq), k/bk] -> int32 [B, Hq, nqb, k/bk if tau else n_e * k/bk]."""
    _need_gpu(samples, indices)
    assert samples.dtype == torch.int32 and samples.is_contiguous() and samples.dim() == 5
    n_e, B, Hq, nqb, kb = samples.shape
    p = HipProblem()
    p.batch, p.n_q_heads, p.n_kv_heads, p.head_dim = B, Hq, 1, 128
    p.q_len, p.max_kv_len, p.k, p.bq, p.bk, p.dtype = q_len, q_len, kb * bk, bq, bk, BF16
    assert (q_len + bq - 1) // bq == nqb
    width = kb if tau else n_e * kb
    if indices is None:
        indices = torch.empty((B, Hq, nqb, width), dtype=torch.int32, device=samples.device)
    assert indices.dtype == torch.int32 and indices.is_contiguous() and indices.numel() == B * Hq * nqb * width
    rc = load().hip_mask_vote(ctypes.byref(p), samples.data_ptr(), n_e, theta_vote, tau, indices.data_ptr(), _stream(samples))
    if rc != 0:
        raise HipAttnError(rc)
    return indices


def hip_mask_ensemble(Q, K, k: int, bq: int, bk: int, n_e: int, theta_vote: int, tau: int, ens_seed: int, ens_r: float,
                      kv_lens=None, page_table=None, max_kv_len=None, flags: int = 0, b_sq: int = 1, b_sk: int = 1,
                      rep_pos: int = 0, top_r: int = 0, workspace: Optional[torch.Tensor] = None,
                      indices: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Ensemble mask: n_e samples of hip_mask_estimate (sample 0 = the plain mask) and the vote over them."""
    _need_gpu(Q, K, kv_lens, page_table, indices, workspace)
    lib = load()
    p = make_problem(Q, K, k, bq, bk, kv_lens, page_table, max_kv_len, flags=flags)
    p.b_sq, p.b_sk, p.rep_pos, p.top_r = b_sq, b_sk, rep_pos, top_r
    p.ens_seed, p.ens_r = ens_seed & 0xffffffff, ens_r
    need = lib.hip_ensemble_workspace_bytes(ctypes.byref(p), n_e)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=Q.device)
    assert workspace.is_contiguous() and workspace.numel() * workspace.element_size() >= need
    p.workspace, p.workspace_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    nqb = (p.q_len + bq - 1) // bq
    width = (k // bk) if tau else n_e * (k // bk)
    if indices is None:
        indices = torch.empty((p.batch, p.n_q_heads, nqb, width), dtype=torch.int32, device=Q.device)
    assert indices.dtype == torch.int32 and indices.is_contiguous() and indices.numel() == p.batch * p.n_q_heads * nqb * width
    rc = lib.hip_mask_ensemble(ctypes.byref(p), Q.data_ptr(), K.data_ptr(), n_e, theta_vote, tau, indices.data_ptr(), _stream(Q))
    if rc != 0:
        raise HipAttnError(rc)
    return indices


STATIC_SCRATCH_BYTES = 8 << 20


def hip_mask_estimate_noalloc(Q, K, k: int, bq: int, bk: int, indices: torch.Tensor, kv_lens=None, page_table=None,
                              max_kv_len=None, flags: int = 0, b_sq: int = 1, b_sk: int = 1, rep_pos: int = 0,
                              top_r: int = 0) -> torch.Tensor:
    """hip_mask_estimate without any allocation: the caller passes `indices`, and the scratch of the top_r option is
    the library's static array (see include/hipattn.h)."""
    _need_gpu(Q, K, kv_lens, page_table, indices)
    p = make_problem(Q, K, k, bq, bk, kv_lens, page_table, max_kv_len, flags=flags)
    p.b_sq, p.b_sk, p.rep_pos, p.top_r = b_sq, b_sk, rep_pos, top_r
    assert indices.dtype == torch.int32 and indices.is_contiguous()
    assert indices.numel() == p.batch * p.n_q_heads * ((p.q_len + bq - 1) // bq) * (k // bk)
    rc = load().hip_mask_estimate_noalloc(ctypes.byref(p), Q.data_ptr(), K.data_ptr(), indices.data_ptr(), _stream(Q))
    if rc != 0:
        raise HipAttnError(rc)
    return indices


def hip_sparse_attn(Q, K, V, indices, k: int, bq: int, bk: int, kv_lens=None, page_table=None,
                    max_kv_len=None, sm_scale: float = 0.0, flags: int = 0,
                    out: Optional[torch.Tensor] = None, n_sink: int = 0, n_window: int = 0,
                    k_backing: Optional[torch.Tensor] = None, v_backing: Optional[torch.Tensor] = None,
                    touched: Optional[torch.Tensor] = None) -> torch.Tensor:
    """O [B, Hq, Tq, d]: attention of every query row over its block's selected keys (plus the first
    n_sink and the n_window most recent keys)."""
    _need_gpu(Q, K, V, indices, kv_lens, page_table, out)
    lib = load()
    assert V.shape == K.shape and V.stride() == K.stride() and V.dtype == K.dtype == Q.dtype
    if out is None:
        out = torch.empty_like(Q)
    assert out.shape == Q.shape and out.dtype == Q.dtype and out.stride(3) == 1
    assert indices.dtype == torch.int32 and indices.is_contiguous()
    p = make_problem(Q, K, k, bq, bk, kv_lens, page_table, max_kv_len, sm_scale, flags, O=out)
    p.n_sink, p.n_window = n_sink, n_window
    _token_bank(p, K, page_table, k_backing, v_backing, touched)
    rc = lib.hip_sparse_attn(ctypes.byref(p), Q.data_ptr(), K.data_ptr(), V.data_ptr(), indices.data_ptr(),
                             out.data_ptr(), _stream(Q))
    if rc != 0:
        raise HipAttnError(rc)
    return out
