"""GPU parity of the ensemble of masks (paper appendix "Ensemble Hierarchical Top-k Approximation"): every sample of
hip_mask_estimate against the oracle's sample, the vote kernel against the oracle's vote, and the whole chain
(samples, vote, sparse attention over the merged list) against the oracle's."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import oracle
import paper_2406_09827_amd as hipattn
from paper_2406_09827_amd import synth
from tests import gpu_util as U

pytestmark = pytest.mark.gpu
S = hipattn.SENTINEL


def _samples_match(w, n_e, seed, r_e, flags=0, units=None, **opts):
    """GPU samples 0 .. n_e-1 against the oracle's, all units or a list; returns the GPU samples [n_e, ...]."""
    x = synth.make_inputs(w, device="cuda", threads=4)
    hx = U.host(x)
    got = []
    moved = 0
    for e in range(n_e):
        U.probes.poison_lds(0xAAAAAAAA)
        idx = torch.full((w.batch, w.n_q_heads, w.n_query_blocks, w.kb), U.UNWRITTEN, dtype=torch.int32, device="cuda")
        hipattn.hip_mask_estimate(x["Q"], x["K"], w.k, w.bq, w.bk, kv_lens=x["kv_lens"], page_table=x["page_table"],
                                  max_kv_len=U._max_len(w, x), flags=flags, indices=idx, ens_sample=e, ens_seed=seed,
                                  ens_r=r_e, **opts)
        torch.cuda.synchronize()
        assert not bool((idx == U.UNWRITTEN).any())
        p = U.oracle_problem(w, x, ens_sample=e, ens_seed=seed, ens_r=r_e, **opts)
        all_u = oracle.all_units(p)
        if units is None:
            sel, us = np.arange(all_u.shape[0]), all_u
        else:
            us = np.asarray(units, dtype=np.int32).reshape(-1, 3)
            sel = (us[:, 0] * p.n_q_heads + us[:, 1]) * p.n_query_blocks + us[:, 2]
        ref = oracle.mask_estimate_units(p, hx["Q"], hx["K"], us)
        g = idx.cpu().numpy().reshape(-1, p.kb)[sel]
        if w.integer:
            bad = np.nonzero((g != ref).any(axis=1))[0]
            assert bad.size == 0, f"sample {e}: {bad.size} units differ, first {us[bad[0]]}"
        else:
            assert U.agreement(g, ref) >= 0.999, (e, U.agreement(g, ref))
        U.check_indices_valid(w, x, g, us)
        if e > 0:
            moved += int((g != got[0].cpu().numpy().reshape(-1, p.kb)[sel]).any())
        got.append(idx)
    if n_e > 1 and r_e > 0:
        assert moved > 0, "no sample differs from the plain mask"
    return x, torch.stack(got)


@pytest.mark.parametrize("integer", [True, False], ids=["int", "normal"])
def test_ensemble_samples_prefill_tuned(integer):
    # 32-row blocks on the direct-to-LDS kernel (k/bk = 128 and 256), a 64-row shape, a paged pool, list rounds
    w = synth.Workload("ens_pre", 1, 4, 2, 128, 6000, 6000, 256, 32, 2, "bf16", rho=0.95, spike_every=1024, integer=integer, seed=701)
    nqb = w.n_query_blocks
    units = [(0, h, qb) for h in range(4) for qb in (3, 9, 17, 40, 77, nqb // 2, nqb - 2, nqb - 1)]
    _samples_match(w, 3, 11, 5.0, units=units)
    _samples_match(synth.scaled(w, k=512, seed=702), 2, 12, 2.5, units=units, rep_pos=2)
    w64 = synth.Workload("ens_pre64", 1, 2, 1, 128, 9000, 9000, 512, 64, 4, "bf16", rho=0.95, integer=integer, seed=703)
    _samples_match(w64, 2, 13, 5.0, units=[(0, h, qb) for h in range(2) for qb in (5, 20, 77, 140)])
    wp = synth.scaled(w, page_size=64, seed=704)
    _samples_match(wp, 2, 14, 5.0, units=units, rep_pos=1)


@pytest.mark.parametrize("integer", [True, False], ids=["int", "normal"])
def test_ensemble_samples_decode_and_generic(integer):
    wd = synth.Workload("ens_dec", 5, 8, 2, 128, 1, 30000, 256, 1, 2, "bf16", rho=0.9, ragged=(700, 30000), integer=integer, seed=705)
    _samples_match(wd, 3, 21, 5.0)
    _samples_match(synth.scaled(wd, page_size=16, seed=706), 2, 22, 5.0, rep_pos=2)
    _samples_match(synth.scaled(wd, batch=1100, kv_len=3000, ragged=(200, 3000), seed=707), 2, 23, 1.5)   # a wave per problem (8800 problems)
    wg = synth.Workload("ens_gen", 2, 2, 1, 64, 900, 900, 48, 16, 2, "fp32", rho=0.9, integer=integer, seed=708)
    _samples_match(wg, 3, 24, 3.0)
    _samples_match(synth.scaled(wd, seed=709), 2, 25, 5.0, flags=hipattn.FORCE_GENERIC)


def _random_sets(rng, n_e, units, kb, span, bk):
    s = np.full((n_e, units, kb), S, dtype=np.int32)
    for e in range(n_e):
        for u in range(units):
            n = int(rng.integers(0, min(kb, span) + 1))
            s[e, u, :n] = np.sort(rng.choice(span, size=n, replace=False)) * bk
    return s


@pytest.mark.parametrize("n_e,kb,span", [(1, 7, 30), (2, 1, 3), (3, 64, 100), (4, 256, 700), (4, 100, 160), (16, 256, 600),
                                         (5, 300, 320), (8, 512, 4000), (16, 3, 5)])
def test_vote_kernel_against_the_oracle(n_e, kb, span):
    rng = np.random.default_rng(n_e * 1000 + kb)
    B, Hq, nqb = 2, 3, 5
    sets = _random_sets(rng, n_e, B * Hq * nqb, kb, span, 2)
    dev = torch.from_numpy(sets.reshape(n_e, B, Hq, nqb, kb)).cuda()
    for theta in sorted({1, 2, max(1, n_e // 2), n_e}):
        for tau in (0, 1):
            U.probes.poison_lds(0x7FC0FFEE)
            width = kb if tau else n_e * kb
            out = torch.full((B, Hq, nqb, width), U.UNWRITTEN, dtype=torch.int32, device="cuda")
            hipattn.hip_mask_vote(dev, theta, tau, bq=4, bk=2, q_len=nqb * 4, indices=out)
            want = oracle.vote(sets, theta, tau)
            assert np.array_equal(out.cpu().numpy().reshape(-1, width), want), (n_e, kb, theta, tau)


def test_vote_argument_errors():
    import ctypes
    lib = hipattn.load()
    p = hipattn.HipProblem()
    p.batch, p.n_q_heads, p.n_kv_heads, p.head_dim = 1, 4, 2, 128
    p.q_len, p.max_kv_len, p.k, p.bq, p.bk, p.dtype = 64, 64, 512, 16, 2, hipattn.BF16
    fake = ctypes.c_void_p(4096)
    assert lib.hip_mask_vote(ctypes.byref(p), fake, 17, 1, 0, fake, None) == -11     # more than 16 sets
    assert lib.hip_mask_vote(ctypes.byref(p), fake, 0, 1, 0, fake, None) == -11
    assert lib.hip_mask_vote(ctypes.byref(p), fake, 4, 0, 0, fake, None) == -11      # theta_vote < 1
    p.k = 2048
    assert lib.hip_mask_vote(ctypes.byref(p), fake, 8, 1, 0, fake, None) == -11      # 8 * 1024 entries
    p.k = 512
    assert lib.hip_mask_vote(ctypes.byref(p), None, 4, 1, 0, fake, None) == -1
    assert lib.hip_mask_ensemble(ctypes.byref(p), fake, fake, 4, 1, 0, fake, None) == -1   # no workspace
    p.workspace, p.workspace_bytes = 4096, 16
    assert lib.hip_mask_ensemble(ctypes.byref(p), fake, fake, 4, 1, 0, fake, None) == -9
    assert lib.hip_ensemble_workspace_bytes(ctypes.byref(p), 4) == 4 * 4 * 4 * 256 * 4
    assert b"ensemble" in lib.hip_strerror(-11)


@pytest.mark.parametrize("tau,theta", [(0, 1), (1, 1), (0, 2)])
def test_ensemble_end_to_end(tau, theta):
    # samples + vote in one call, then sparse attention over the merged list, against the oracle's chain
    n_e, seed, r_e = 4, 31, 5.0
    for w in (synth.Workload("ens_e2e", 1, 4, 2, 128, 5000, 5000, 256, 32, 2, "bf16", rho=0.95, integer=True, seed=711),
              synth.Workload("ens_e2e_dec", 4, 8, 2, 128, 1, 20000, 256, 1, 2, "bf16", rho=0.9, ragged=(3000, 20000),
                             page_size=64, integer=True, seed=712)):
        x = synth.make_inputs(w, device="cuda", threads=4)
        hx = U.host(x)
        kw = dict(kv_lens=x["kv_lens"], page_table=x["page_table"], max_kv_len=U._max_len(w, x))
        merged = hipattn.hip_mask_ensemble(x["Q"], x["K"], w.k, w.bq, w.bk, n_e, theta, tau, seed, r_e, **kw)
        width = merged.shape[-1]
        refs = np.stack([oracle.mask_estimate(U.oracle_problem(w, x, ens_sample=e, ens_seed=seed, ens_r=r_e), hx["Q"], hx["K"])
                         for e in range(n_e)])
        want = oracle.vote(refs, theta, tau)
        assert np.array_equal(merged.cpu().numpy(), want)
        if theta == 1:   # the union holds the plain mask
            plain = refs[0]
            assert all(set(a[a != S]) <= set(b[b != S]) or tau for a, b in zip(plain.reshape(-1, w.kb), want.reshape(-1, width)))
        out = hipattn.hip_sparse_attn(x["Q"], x["K"], x["V"], merged, width * w.bk, w.bq, w.bk, **kw)
        pm = replace(U.oracle_problem(w, x), k=width * w.bk)
        o_ref = oracle.sparse_attn(pm, hx["Q"], hx["K"], hx["V"], want)
        U.check_output(out.float().cpu().numpy(), o_ref, w.dtype)
