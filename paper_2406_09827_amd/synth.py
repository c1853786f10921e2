"""Seeded synthetic inputs for the HiP hot path.

This module holds NO arithmetic of the method: it only draws random tensors with
the structure of the paper's workloads (attention locality: keys that are close
in the sequence are similar, Sec. 4 "Observation"; a few heavy-hitter tokens),
rounds them ONCE to the workload's dtype and hands the same rounded values to
whoever asks - the GPU path and the CPU oracle both consume them.

Recipe
------
K, V : independent AR(1) chains along the sequence for every (sequence, kv head,
       channel): x_0 = e_0, x_t = rho * x_{t-1} + e_t, e ~ N(0,1) (not variance
       normalised).  K and V use different random streams.
Q    : i.i.d. N(0,1).
spikes: after the recursion, key rows at t in {P*i, P*i+1} (one key block) are
       multiplied by `spike_scale` for every i >= 0 (P = `spike_every`).
integer variant: Q, K, V i.i.d. uniform on {-4,...,4}/8 - exact in bf16/fp32 and
       every dot product is exact in fp32 in any summation order.
ragged: kv_lens ~ U{lo..hi}; paged: K/V live in a pool [n_pages, Hkv, page, d]
       addressed through a random permutation page table.
Random numbers come from numpy's counter-based Philox generator keyed by
(seed, tensor id, sequence, kv head), so any slice can be regenerated alone.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
from typing import Dict, Optional, Tuple

import numpy as np
import torch
from scipy.signal import lfilter

SEED_BASE = 0x48695000


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    q_len: int            # query rows per sequence (== kv_len for prefill, 1 for decode)
    kv_len: int           # context length (max over sequences when ragged)
    k: int
    bq: int
    bk: int
    dtype: str            # "fp32" | "bf16"
    rho: float = 0.9
    spike_every: int = 0
    spike_scale: float = 4.0
    ragged: Optional[Tuple[int, int]] = None   # (lo, hi) inclusive
    page_size: int = 0                          # 0 = contiguous [B,Hkv,T,d]
    integer: bool = False
    seed: int = SEED_BASE

    @property
    def kb(self) -> int:
        return self.k // self.bk

    @property
    def n_query_blocks(self) -> int:
        return (self.q_len + self.bq - 1) // self.bq

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "fp32" else torch.bfloat16


# The five workloads of the benchmark description, plus the integer variant of the first.
C1 = Workload("c1_prefill_1k_fp32", 1, 1, 1, 64, 1024, 1024, 128, 16, 2, "fp32", rho=0.9, seed=SEED_BASE + 1)
C1_INT = replace(C1, name="c1_prefill_1k_fp32_int", integer=True)
C2 = Workload("c2_prefill_32k_bf16", 1, 32, 8, 128, 32768, 32768, 512, 32, 2, "bf16", rho=0.95,
              spike_every=4096, seed=SEED_BASE + 2)
C2_INT = replace(C2, name="c2_prefill_32k_bf16_int", integer=True)
C3 = Workload("c3_decode_128k_bf16", 32, 32, 8, 128, 1, 131072, 512, 1, 2, "bf16", rho=0.9, seed=SEED_BASE + 3)
C4 = Workload("c4_prefill_1m_bf16", 1, 32, 8, 128, 1048576, 1048576, 2048, 64, 4, "bf16", rho=0.95,
              seed=SEED_BASE + 4)
C5 = Workload("c5_ragged_paged_decode_bf16", 256, 32, 8, 128, 1, 65536, 512, 1, 2, "bf16", rho=0.9,
              ragged=(8192, 65536), page_size=64, seed=SEED_BASE + 5)
# The two latency workloads of the paper's block-size ablation (LLaMA-2-7B-32k-shaped layer: 32 MHA heads,
# d=128, T=12k, batch 96, k=512, mask re-estimated every step): single-query decode and decode with 32
# query rows per sequence (speculative decoding).
PD = Workload("pd_paper_decode_12k_bf16", 96, 32, 32, 128, 1, 12288, 512, 1, 2, "bf16", rho=0.9, seed=SEED_BASE + 6)
PS = Workload("ps_paper_specdec_12k_bf16", 96, 32, 32, 128, 32, 12288, 512, 32, 2, "bf16", rho=0.9, seed=SEED_BASE + 7)
WORKLOADS = {w.name.split("_")[0]: w for w in (C1, C2, C3, C4, C5, PD, PS)}


def scaled(w: Workload, **kw) -> Workload:
    """A smaller or altered copy of a workload (tests use reduced sizes of the same recipe)."""
    return replace(w, **kw)


def _rng(seed: int, tensor_id: int, b: int = 0, h: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed & (2**64 - 1), (tensor_id << 40) | (b << 16) | h]))


def _round(x: np.ndarray, w: Workload) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    return t.to(w.torch_dtype)


def _int_values(rng: np.random.Generator, shape) -> np.ndarray:
    return rng.integers(-4, 5, size=shape).astype(np.float32) / 8.0


def kv_lens_of(w: Workload) -> Optional[np.ndarray]:
    if w.ragged is None:
        return None
    lo, hi = w.ragged
    return _rng(w.seed, 7).integers(lo, hi + 1, size=w.batch).astype(np.int32)


def kv_sequence(w: Workload, which: str, b: int, h: int, length: int) -> torch.Tensor:
    """[length, d] rows of K ("k") or V ("v") of sequence b, kv head h, rounded to the dtype."""
    tid = 1 if which == "k" else 2
    rng = _rng(w.seed, tid, b, h)
    if w.integer:
        x = _int_values(rng, (length, w.head_dim))
    else:
        eps = rng.standard_normal((length, w.head_dim), dtype=np.float32)
        x = lfilter([1.0], [1.0, -w.rho], eps.astype(np.float64), axis=0).astype(np.float32)
        if which == "k" and w.spike_every > 0:
            for t0 in range(0, length, w.spike_every):
                x[t0:t0 + 2] *= w.spike_scale
    return _round(x, w)


def q_rows(w: Workload, b: int, h: int) -> torch.Tensor:
    """[q_len, d] query rows of sequence b, query head h."""
    rng = _rng(w.seed, 3, b, h)
    if w.integer:
        x = _int_values(rng, (w.q_len, w.head_dim))
    else:
        x = rng.standard_normal((w.q_len, w.head_dim), dtype=np.float32)
    return _round(x, w)


def make_inputs(w: Workload, device="cpu", threads: int = 8) -> Dict[str, object]:
    """All tensors of a workload on `device`, generated slice by slice.

    Returns a dict with Q [B,Hq,Tq,d]; K, V either [B,Hkv,T,d] or, when paged, the pool
    [n_pages,Hkv,page,d]; kv_lens (int32 [B] or None); page_table (int32 [B,max_pages] or None).
    Rows of a contiguous K/V beyond a sequence's kv_len are zero.
    """
    dt = w.torch_dtype
    lens = kv_lens_of(w)
    out: Dict[str, object] = {"kv_lens": None, "page_table": None}
    Q = torch.empty((w.batch, w.n_q_heads, w.q_len, w.head_dim), dtype=dt, device=device)

    def fill_q(bh):
        b, h = bh
        Q[b, h].copy_(q_rows(w, b, h))

    jobs_q = [(b, h) for b in range(w.batch) for h in range(w.n_q_heads)]

    if w.page_size:
        ps = w.page_size
        seq_len = lens if lens is not None else np.full(w.batch, w.kv_len, np.int32)
        n_pages_seq = (seq_len.astype(np.int64) + ps - 1) // ps
        n_pages = int(n_pages_seq.sum())
        perm = _rng(w.seed, 8).permutation(n_pages).astype(np.int32)
        max_pages = int(n_pages_seq.max())
        table = np.zeros((w.batch, max_pages), dtype=np.int32)
        off = 0
        for b in range(w.batch):
            table[b, :n_pages_seq[b]] = perm[off:off + n_pages_seq[b]]
            off += int(n_pages_seq[b])
        K = torch.zeros((n_pages, w.n_kv_heads, ps, w.head_dim), dtype=dt, device=device)
        V = torch.zeros_like(K)

        def fill_kv(bh):
            b, h = bh
            n, npg = int(seq_len[b]), int(n_pages_seq[b])
            pages = torch.from_numpy(table[b, :npg].astype(np.int64)).to(device)
            for which, dst in (("k", K), ("v", V)):
                x = kv_sequence(w, which, b, h, n)
                pad = torch.zeros((npg * ps, w.head_dim), dtype=dt)
                pad[:n] = x
                dst[pages, h] = pad.view(npg, ps, w.head_dim).to(device)

        out["page_table"] = torch.from_numpy(table).to(device)
    else:
        K = torch.zeros((w.batch, w.n_kv_heads, w.kv_len, w.head_dim), dtype=dt, device=device)
        V = torch.zeros_like(K)

        def fill_kv(bh):
            b, h = bh
            n = int(lens[b]) if lens is not None else w.kv_len
            K[b, h, :n].copy_(kv_sequence(w, "k", b, h, n))
            V[b, h, :n].copy_(kv_sequence(w, "v", b, h, n))

    jobs_kv = [(b, h) for b in range(w.batch) for h in range(w.n_kv_heads)]
    if threads > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill_q, jobs_q))
            list(ex.map(fill_kv, jobs_kv))
    else:
        for j in jobs_q:
            fill_q(j)
        for j in jobs_kv:
            fill_kv(j)
    if lens is not None:
        out["kv_lens"] = torch.from_numpy(lens).to(device)
    out.update(Q=Q, K=K, V=V)
    return out


def token_bank(x: Dict[str, object], w: Workload, resident_frac: float, host_backing: bool = False,
               poison: float = 7.0) -> Dict[str, object]:
    """Re-houses a paged input as a bank of resident pages plus a backing pool (the layout of the paper's
    KV cache offloading, Sec. 3.3): every used page is resident with probability `resident_frac`.

    Returns a copy of `x` in which K, V are the bank [n_resident, Hkv, page, d] (resident pages in random order),
    `k_backing`, `v_backing` the full pools (in pinned host memory with `host_backing`), and `page_table` holds
    the bank slot (>= 0) of a resident page and -(backing page) - 1 of any other.  With `poison`, the backing
    copies of the resident pages are overwritten with that value, so a look-up that goes to the wrong pool shows.
    """
    assert w.page_size and x["page_table"] is not None
    K, V = x["K"], x["V"]
    table = x["page_table"].cpu().numpy().astype(np.int64)
    lens = x["kv_lens"].cpu().numpy() if x["kv_lens"] is not None else np.full(w.batch, w.kv_len)
    n_used = (lens.astype(np.int64) + w.page_size - 1) // w.page_size
    used = np.arange(table.shape[1])[None, :] < n_used[:, None]
    rng = _rng(w.seed, 9)
    resident = used & (rng.random(table.shape) < resident_frac)
    pages = table[resident]                       # backing pages that get a bank slot
    slots = rng.permutation(pages.size)
    new_table = np.where(used, -table - 1, 0)
    new_table[resident] = slots
    order = np.empty(max(pages.size, 1), dtype=np.int64)
    order[:] = pages[0] if pages.size else 0
    order[slots] = pages
    sel = torch.from_numpy(order).to(K.device)
    out = dict(x)
    out["K"], out["V"] = K[sel].contiguous(), V[sel].contiguous()
    kb_, vb_ = K.clone(), V.clone()
    if poison and pages.size:
        kb_[sel] = poison
        vb_[sel] = poison
    if not pages.size:
        out["K"].fill_(poison)
        out["V"].fill_(poison)
    if host_backing:
        kb_, vb_ = kb_.cpu().pin_memory(), vb_.cpu().pin_memory()
    out["k_backing"], out["v_backing"] = kb_, vb_
    out["page_table"] = torch.from_numpy(new_table.astype(np.int32)).to(K.device)
    out["resident"] = resident
    return out
