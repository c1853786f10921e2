"""ctypes front end of the CPU oracle (``hip_oracle.c``).

TEST INFRASTRUCTURE: only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package.  It shares nothing
with the GPU library and never imports it.

The wrapper only marshals numpy arrays; every step of the method (Alg. 1,
Eq. 1-5 of the paper) is in the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hip_oracle.c")
_LIB = os.path.join(_HERE, "libhip_oracle.so")
SENTINEL = np.iinfo(np.int32).max


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over independent units)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Problem(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("q_len", ctypes.c_int32), ("max_kv_len", ctypes.c_int32),
        ("k", ctypes.c_int32), ("bq", ctypes.c_int32), ("bk", ctypes.c_int32),
        ("kv_lens", ctypes.c_void_p), ("page_table", ctypes.c_void_p),
        ("page_size", ctypes.c_int32), ("max_pages", ctypes.c_int32),
        ("n_threads", ctypes.c_int32), ("n_sink", ctypes.c_int32), ("n_window", ctypes.c_int32),
        ("b_sq", ctypes.c_int32), ("b_sk", ctypes.c_int32), ("rep_pos", ctypes.c_int32),
        ("top_r", ctypes.c_int32),
        ("k_backing", ctypes.c_void_p), ("v_backing", ctypes.c_void_p), ("touched", ctypes.c_void_p),
        ("ens_sample", ctypes.c_int32), ("ens_seed", ctypes.c_uint32), ("ens_r", ctypes.c_float),
    ]


class _Stats(ctypes.Structure):
    _fields_ = [("rounds", ctypes.c_int32), ("first_chunk_max", ctypes.c_int32),
                ("reps_scored", ctypes.c_int64)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_hip_mask_estimate_units.restype = ctypes.c_int
        _lib.oracle_hip_sparse_attn_units.restype = ctypes.c_int
        _lib.oracle_hip_sparse_attn_units.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int64, ctypes.c_void_p, ctypes.c_double, ctypes.c_void_p]
        _lib.oracle_hip_mask_estimate_units.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
        _lib.oracle_hip_vote.restype = ctypes.c_int
        _lib.oracle_hip_vote.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32,
                                         ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p]
    return _lib


@dataclass
class Problem:
    """Shape of one HiP attention call (same meaning as the paper's T, k, b_q, b_k)."""
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    q_len: int
    max_kv_len: int
    k: int
    bq: int
    bk: int
    kv_lens: Optional[np.ndarray] = None      # int32 [batch]
    page_table: Optional[np.ndarray] = None   # int32 [batch, max_pages]
    page_size: int = 0
    n_threads: int = 1
    n_sink: int = 0      # sparse attention: the first n_sink keys are always attended
    n_window: int = 0    # sparse attention: the n_window most recent keys are always attended
    b_sq: int = 1        # mask estimation: score every b_sq-th row of the query block
    b_sk: int = 1        # mask estimation: score every b_sk-th key of the representative block
    rep_pos: int = 0     # mask estimation: representative block of a branch: 0 centre, 1 first, 2 last
    top_r: int = 0       # mask estimation: channels of largest |q| used per query row (0 = all)
    # token bank (Sec. 3.3): pools read for negative page-table entries (entry e names page -e-1), same layout
    # as K / V; touched [batch, max_pages] uint8 receives 1 for every logical page a call reads
    k_backing: Optional[np.ndarray] = None
    v_backing: Optional[np.ndarray] = None
    touched: Optional[np.ndarray] = None
    # ensemble sample (appendix "Ensemble Hierarchical Top-k Approximation"): 0 = the plain mask; e > 0 adds
    # ens_r * u, u a counter-based uniform on [-1, 1), to the scores of the middle round
    ens_sample: int = 0
    ens_seed: int = 0
    ens_r: float = 0.0

    @property
    def kb(self) -> int:
        return self.k // self.bk

    @property
    def n_query_blocks(self) -> int:
        return (self.q_len + self.bq - 1) // self.bq

    def _c(self):
        keep = []
        p = _Problem(self.batch, self.n_q_heads, self.n_kv_heads, self.head_dim, self.q_len,
                     self.max_kv_len, self.k, self.bq, self.bk, None, None, 0, 0, self.n_threads,
                     self.n_sink, self.n_window, self.b_sq, self.b_sk, self.rep_pos, self.top_r)
        p.ens_sample, p.ens_seed, p.ens_r = self.ens_sample, self.ens_seed & 0xffffffff, self.ens_r
        if self.kv_lens is not None:
            a = np.ascontiguousarray(self.kv_lens, dtype=np.int32)
            assert a.shape == (self.batch,)
            keep.append(a)
            p.kv_lens = a.ctypes.data
        if self.page_table is not None:
            a = np.ascontiguousarray(self.page_table, dtype=np.int32)
            assert a.ndim == 2 and a.shape[0] == self.batch
            keep.append(a)
            p.page_table = a.ctypes.data
            p.page_size = self.page_size
            p.max_pages = a.shape[1]
        for name in ("k_backing", "v_backing"):
            x = getattr(self, name)
            if x is not None:
                assert self.page_table is not None and x.dtype == np.float32 and x.flags.c_contiguous
                assert x.ndim == 4 and x.shape[1:] == (self.n_kv_heads, self.page_size, self.head_dim), x.shape
                assert -int(np.min(self.page_table)) - 1 < x.shape[0]
                keep.append(x)
                setattr(p, name, x.ctypes.data)
        if self.touched is not None:
            t = self.touched
            assert self.page_table is not None and t.dtype == np.uint8 and t.flags.c_contiguous
            assert t.shape == self.page_table.shape
            p.touched = t.ctypes.data
        return p, keep


def _f32(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _check_shapes(p: Problem, Q, K, V=None):
    assert Q.shape == (p.batch, p.n_q_heads, p.q_len, p.head_dim), Q.shape
    for X in (K, V):
        if X is None:
            continue
        if p.page_table is not None:
            assert X.ndim == 4 and X.shape[1:] == (p.n_kv_heads, p.page_size, p.head_dim), X.shape
            assert int(np.max(p.page_table)) < X.shape[0]
        else:
            assert X.shape == (p.batch, p.n_kv_heads, p.max_kv_len, p.head_dim), X.shape


def all_units(p: Problem) -> np.ndarray:
    b, h, q = np.meshgrid(np.arange(p.batch), np.arange(p.n_q_heads), np.arange(p.n_query_blocks),
                          indexing="ij")
    return np.stack([b.ravel(), h.ravel(), q.ravel()], axis=1).astype(np.int32)


def mask_estimate_units(p: Problem, Q, K, units, with_stats: bool = False):
    """Indices [n_units, kb] (and per-unit stats) for the listed (b, h, qb) units."""
    Q, K = _f32(Q), _f32(K)
    _check_shapes(p, Q, K)
    units = np.ascontiguousarray(units, dtype=np.int32).reshape(-1, 3)
    n = units.shape[0]
    out = np.empty((n, p.kb), dtype=np.int32)
    stats = (_Stats * max(n, 1))() if with_stats else None
    cp, keep = p._c()
    rc = lib().oracle_hip_mask_estimate_units(
        ctypes.byref(cp), Q.ctypes.data, K.ctypes.data, units.ctypes.data, n, out.ctypes.data,
        ctypes.cast(stats, ctypes.c_void_p) if with_stats else None)
    if rc != 0:
        raise ValueError("oracle rejected the problem description")
    del keep
    if with_stats:
        st = [dict(rounds=s.rounds, first_chunk_max=s.first_chunk_max, reps_scored=s.reps_scored)
              for s in stats[:n]]
        return out, st
    return out


def mask_estimate(p: Problem, Q, K) -> np.ndarray:
    """Indices [batch, n_q_heads, n_query_blocks, kb] int32 (Alg. 1 output)."""
    out = mask_estimate_units(p, Q, K, all_units(p))
    return out.reshape(p.batch, p.n_q_heads, p.n_query_blocks, p.kb)


def sparse_attn_units(p: Problem, Q, K, V, units, idx, sm_scale: float = 0.0) -> np.ndarray:
    """O [n_units, bq, d] float64 for the listed units; idx is [n_units, kb]."""
    Q, K, V = _f32(Q), _f32(K), _f32(V)
    _check_shapes(p, Q, K, V)
    units = np.ascontiguousarray(units, dtype=np.int32).reshape(-1, 3)
    n = units.shape[0]
    idx = np.ascontiguousarray(idx, dtype=np.int32).reshape(n, p.kb)
    O = np.zeros((n, p.bq, p.head_dim), dtype=np.float64)
    cp, keep = p._c()
    rc = lib().oracle_hip_sparse_attn_units(
        ctypes.byref(cp), Q.ctypes.data, K.ctypes.data, V.ctypes.data, units.ctypes.data, n,
        idx.ctypes.data, float(sm_scale), O.ctypes.data)
    if rc != 0:
        raise ValueError("oracle rejected the problem description")
    del keep
    return O


def sparse_attn(p: Problem, Q, K, V, indices, sm_scale: float = 0.0) -> np.ndarray:
    """O [batch, n_q_heads, q_len, d] float64 (Eq. 2 with the mask given by `indices`)."""
    units = all_units(p)
    idx = np.ascontiguousarray(indices, dtype=np.int32).reshape(units.shape[0], p.kb)
    Ou = sparse_attn_units(p, Q, K, V, units, idx, sm_scale)
    nqb = p.n_query_blocks
    O = Ou.reshape(p.batch, p.n_q_heads, nqb * p.bq, p.head_dim)[:, :, :p.q_len, :]
    return np.ascontiguousarray(O)


def vote(samples, theta_vote: int, tau: int) -> np.ndarray:
    """Ensemble vote: samples [n_e, ..., kb] index sets -> [..., kb if tau else n_e * kb] (see hip_oracle.c)."""
    samples = np.ascontiguousarray(samples, dtype=np.int32)
    n_e, kb = samples.shape[0], samples.shape[-1]
    lead = samples.shape[1:-1]
    n_units = int(np.prod(lead)) if lead else 1
    width = kb if tau else n_e * kb
    out = np.empty((n_units, width), dtype=np.int32)
    rc = lib().oracle_hip_vote(samples.ctypes.data, n_e, n_units, kb, int(theta_vote), int(tau), out.ctypes.data)
    if rc != 0:
        raise ValueError("oracle rejected the vote description")
    return out.reshape(*lead, width)


def problem_for(w, x, n_threads: int = 8, **options) -> Problem:
    """The Problem of a seeded workload description `w` (fields batch, n_q_heads, ..., page_size) and its
    generated inputs `x` (a dict with "kv_lens" and "page_table", tensors or None); `options` are Problem's
    optional fields (n_sink, n_window, b_sq, b_sk, rep_pos, top_r)."""
    lens = x["kv_lens"].cpu().numpy() if x["kv_lens"] is not None else None
    table = x["page_table"].cpu().numpy() if x["page_table"] is not None else None
    return Problem(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.q_len, w.kv_len, w.k, w.bq, w.bk,
                   kv_lens=lens, page_table=table, page_size=w.page_size, n_threads=n_threads, **options)


def host_arrays(x) -> dict:
    """Q, K, V of generated inputs as float32 numpy arrays (the dtype-rounded values, exactly)."""
    return {n: x[n].float().cpu().numpy() for n in ("Q", "K", "V")}
