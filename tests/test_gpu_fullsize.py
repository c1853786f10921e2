"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times:
sampled (sequence, head, query block) units against the oracle, plus invariants over the
whole result."""
import os

import numpy as np
import pytest
import torch

import paper_2406_09827_amd as hipattn
from paper_2406_09827_amd import synth
from tests import gpu_util as U

pytestmark = pytest.mark.gpu


def _whole_result_invariants(w, x, idx):
    """ascending / multiple of bk / causal / sentinel-suffix checks over every unit, on the GPU."""
    kb, bk = w.kb, w.bk
    B, H, NQB = w.batch, w.n_q_heads, w.n_query_blocks
    lens = x["kv_lens"].long() if x["kv_lens"] is not None else torch.full((B,), w.kv_len, device="cuda")
    qb = torch.arange(NQB, device="cuda")
    last_row = torch.minimum((qb + 1) * w.bq, torch.tensor(w.q_len, device="cuda")) - 1
    L = torch.minimum(lens[:, None], lens[:, None] - w.q_len + last_row[None, :] + 1).clamp(min=0)   # [B, NQB]
    Tb = (L + bk - 1) // bk
    nv = torch.clamp(Tb, max=kb)[:, None, :, None]                                                    # [B,1,NQB,1]
    j = torch.arange(kb, device="cuda")[None, None, None, :]
    valid = j < nv
    i64 = idx.long()
    assert bool(((i64 == hipattn.SENTINEL) | valid).all()) and bool(((i64 != hipattn.SENTINEL) | ~valid).all())
    assert bool(((i64 % bk == 0) | ~valid).all())
    assert bool(((i64 < L[:, None, :, None]) | ~valid).all())
    inc = (i64[..., 1:] > i64[..., :-1]) | ~valid[..., 1:].expand_as(i64[..., 1:])
    assert bool(inc.all())


def _sampled_units(w, n, seed):
    rng = np.random.default_rng(seed)
    nqb = w.n_query_blocks
    units = set()
    if nqb > 1:
        for qb in (0, nqb // 2, nqb - 1):
            units.add((0, int(rng.integers(w.n_q_heads)), qb))
    while len(units) < n:
        units.add((int(rng.integers(w.batch)), int(rng.integers(w.n_q_heads)), int(rng.integers(nqb))))
    return sorted(units)


def _fullsize(w, n_units, seed):
    x = synth.make_inputs(w, device="cuda", threads=16)
    idx = U.gpu_mask(w, x)
    out = U.gpu_attn(w, x, idx)
    torch.cuda.synchronize()
    U.every_unit_written(idx, out)
    _whole_result_invariants(w, x, idx)
    assert bool(torch.isfinite(out.float()).all())
    units = np.array(_sampled_units(w, n_units, seed), dtype=np.int32)
    p = U.oracle_problem(w, x)
    # only the sampled sequences / heads go to the host
    import oracle
    idx_g = idx.cpu().numpy().reshape(-1, w.kb)
    nqb = w.n_query_blocks
    worst, agree, total = 0.0, 0, 0
    for (b, h, qb) in units:
        hk = h // (w.n_q_heads // w.n_kv_heads)
        table = None
        if w.page_size:
            # the sequence's own pages, in logical order, as a pool of their own
            n_pages = -(-int(p.kv_lens[b] if p.kv_lens is not None else w.kv_len) // w.page_size)
            pages = x["page_table"][b, :n_pages].long()
            table = np.arange(n_pages, dtype=np.int32)[None]
        sub = oracle.Problem(1, 1, 1, w.head_dim, w.q_len, w.kv_len, w.k, w.bq, w.bk,
                             kv_lens=None if p.kv_lens is None else p.kv_lens[b:b + 1],
                             page_table=table, page_size=w.page_size)
        Q = x["Q"][b:b + 1, h:h + 1].float().cpu().numpy()
        if w.page_size:
            K = x["K"][pages, hk:hk + 1].float().cpu().numpy()
            V = x["V"][pages, hk:hk + 1].float().cpu().numpy()
        else:
            K = x["K"][b:b + 1, hk:hk + 1].float().cpu().numpy()
            V = x["V"][b:b + 1, hk:hk + 1].float().cpu().numpy()
        u1 = np.array([[0, 0, qb]], dtype=np.int32)
        ref = oracle.mask_estimate_units(sub, Q, K, u1)[0]
        got = idx_g[(b * w.n_q_heads + h) * nqb + qb]
        if w.integer:
            assert np.array_equal(got, ref), (b, h, qb)
        agree += int((got == ref).sum()); total += got.size
        o_ref = oracle.sparse_attn_units(sub, Q, K, V, u1, got[None])[0]
        r0 = qb * w.bq
        n = min(w.bq, w.q_len - r0)
        worst = max(worst, U.check_output(out[b, h, r0:r0 + n].float().cpu().numpy(), o_ref[:n], w.dtype))
    assert agree / total >= 0.999, agree / total
    return agree / total, worst


@pytest.mark.parametrize("integer", [True, False], ids=["int", "normal"])
def test_c2_full_size(integer):
    w = synth.C2_INT if integer else synth.C2
    agr, err = _fullsize(w, 40, seed=3)
    print(f"C2 full size: agreement {agr:.6f}, max |dO| {err:.3e}")


@pytest.mark.parametrize("integer", [True, False], ids=["int", "normal"])
def test_c3_full_size(integer):
    w = synth.scaled(synth.C3, integer=integer)
    agr, err = _fullsize(w, 24, seed=4)
    print(f"C3 full size: agreement {agr:.6f}, max |dO| {err:.3e}")


def test_c5_ragged_paged_quarter_batch():
    # the ragged, paged decode workload at a quarter of its batch (64 sequences, ~4.7 GB of KV: 32-bit page offsets)
    w = synth.scaled(synth.C5, batch=64)
    agr, err = _fullsize(w, 24, seed=5)
    print(f"C5/4: agreement {agr:.6f}, max |dO| {err:.3e}")


def test_c5_full_batch():
    # the ragged, paged decode workload as bench.py launches it: 256 sequences = 8192 (sequence, head) problems
    # (a workgroup per problem; ~18 GiB pools, 64-bit page offsets); only the sampled sequences' rows go to the host
    agr, err = _fullsize(synth.C5, 32, seed=9)
    print(f"C5 full batch: agreement {agr:.6f}, max |dO| {err:.3e}")


def test_c2_shape_at_128k_and_256k():
    # all eight KV heads at 128k / 256k tokens: the launches work on 4, 2 or 1 (sequence, kv head) groups at a
    # time (placement by cache capacity), with integer-valued inputs so that the indices are exact
    for T, n in ((131072, 16), (262144 + 96, 10)):   # the second: workgroup counts that do not divide evenly over the XCDs
        w = synth.scaled(synth.C2_INT, q_len=T, kv_len=T)
        agr, err = _fullsize(w, n, seed=8)
        print(f"C2@{T}: agreement {agr:.6f}, max |dO| {err:.3e}")


def test_c4_shape_at_128k():
    # the million-token workload's shape (k=2048, bq=64, bk=4) at T = 131072, 8 query heads
    w = synth.scaled(synth.C4, q_len=131072, kv_len=131072, n_q_heads=8, n_kv_heads=2)
    agr, err = _fullsize(w, 16, seed=6)
    print(f"C4@128k: agreement {agr:.6f}, max |dO| {err:.3e}")


@pytest.mark.skipif(os.environ.get("HIPATTN_SKIP_C4_FULL") == "1", reason="HIPATTN_SKIP_C4_FULL=1")
def test_c4_full_size():
    # the million-token workload as bench.py launches it (about 20 s, most of it input generation)
    agr, err = _fullsize(synth.C4, 12, seed=7)
    print(f"C4 full size: agreement {agr:.6f}, max |dO| {err:.3e}")
