"""ctypes binding of libhipattn_aux.so: the test and measurement aids of include/hipattn_aux.h.

Kept apart from the product binding: the GPU tests poison the LDS before every call, the benchmark
measures the ceilings of the GPU it runs on.  No step of the method lives here.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhipattn_aux.so")
EXPORTS = ("hip_attn_poison_lds", "hip_attn_probe_copy", "hip_attn_probe_read", "hip_attn_probe_mfma",
           "hip_attn_probe_gather")
PROBE_READ_WORDS = 256 * 32 * 256

_lib = None


def load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built; run __graft_entry__.build()")
        lib = ctypes.CDLL(LIB_PATH)
        for n in EXPORTS:
            getattr(lib, n).restype = ctypes.c_int
        lib.hip_attn_poison_lds.argtypes = [ctypes.c_uint32, ctypes.c_void_p]
        lib.hip_attn_probe_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        lib.hip_attn_probe_read.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        lib.hip_attn_probe_mfma.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p]
        lib.hip_attn_probe_gather.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32,
                                              ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p]
        _lib = lib
    return _lib


def _check(rc: int) -> None:
    if rc != 0:
        raise RuntimeError(f"hipattn_aux error {rc}")


def _stream(t: torch.Tensor) -> int:
    return torch.cuda.current_stream(t.device).cuda_stream


def _nbytes(t: torch.Tensor) -> int:
    return t.numel() * t.element_size()


def poison_lds(pattern: int = 0xAAAAAAAA) -> None:
    """Overwrite the LDS of every compute unit."""
    _check(load().hip_attn_poison_lds(pattern, torch.cuda.current_stream().cuda_stream))


def probe_copy(dst: torch.Tensor, src: torch.Tensor) -> None:
    """One copy kernel src -> dst."""
    assert dst.is_cuda and src.is_cuda and _nbytes(dst) == _nbytes(src) and dst.is_contiguous() and src.is_contiguous()
    _check(load().hip_attn_probe_copy(dst.data_ptr(), src.data_ptr(), _nbytes(src), _stream(src)))


def probe_read(out: torch.Tensor, src: torch.Tensor) -> None:
    """One read-only sweep of src; out (int32 [PROBE_READ_WORDS]) receives per-lane XORs."""
    assert out.is_cuda and src.is_cuda and out.dtype == torch.int32 and out.is_contiguous()
    assert out.numel() >= PROBE_READ_WORDS and src.is_contiguous()
    _check(load().hip_attn_probe_read(out.data_ptr(), src.data_ptr(), _nbytes(src), _stream(src)))


def probe_mfma(out: torch.Tensor, workgroups: int, iters: int) -> float:
    """Back-to-back bf16 MFMAs; returns the flops the launch performs."""
    assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous() and out.numel() >= workgroups * 256
    _check(load().hip_attn_probe_mfma(out.data_ptr(), workgroups, iters, _stream(out)))
    return workgroups * 4 * iters * 4 * 2.0 * 32 * 32 * 16


def probe_gather(out: torch.Tensor, src: torch.Tensor, slices: int, run_rows: int, workgroups: int, tiles: int) -> int:
    """The attention kernels' gather pattern over `src`; returns the bytes the launch gathers."""
    assert out.is_cuda and src.is_cuda and out.dtype == torch.int32 and out.is_contiguous() and src.is_contiguous()
    assert out.numel() >= workgroups * 256
    _check(load().hip_attn_probe_gather(out.data_ptr(), src.data_ptr(), _nbytes(src), slices, run_rows, workgroups, tiles,
                                        _stream(src)))
    return workgroups * 4 * tiles * 8192
