"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle."""
import numpy as np
import pytest
import paper_2406_09827_amd as hipattn
import torch

from paper_2406_09827_amd import synth, FORCE_GENERIC
from tests import gpu_util as U

pytestmark = pytest.mark.gpu

FLAG_SETS = [pytest.param(FORCE_GENERIC, id="generic"), pytest.param(0, id="tuned")]


@pytest.mark.parametrize("flags", FLAG_SETS)
def test_c1_integer_bit_exact(flags):
    U.run_case(synth.C1_INT, flags)


@pytest.mark.parametrize("flags", FLAG_SETS)
def test_c1_normal(flags):
    agr, err = U.run_case(synth.C1, flags)
    print(f"c1 agreement {agr:.6f} max err {err:.3e}")


@pytest.mark.parametrize("flags", FLAG_SETS)
@pytest.mark.parametrize("integer", [True, False], ids=["int", "normal"])
def test_c2_shape_reduced(flags, integer):
    # C2's head layout, block sizes and k, at T = 4096 + a ragged tail (several tiles, short last block)
    w = synth.scaled(synth.C2, q_len=4096 + 40, kv_len=4096 + 40, n_q_heads=8, n_kv_heads=2, spike_every=1024,
                     integer=integer)
    rng = np.random.default_rng(0)
    nqb = w.n_query_blocks
    qbs = sorted(set([0, 7, 8, 9, 15, 16, 17, 31, 32, 33, 64, nqb - 2, nqb - 1] + rng.integers(0, nqb, 12).tolist()))
    units = [(0, h, qb) for h in range(w.n_q_heads) for qb in qbs]
    agr, err = U.run_case(w, flags, units=units)
    print(f"c2-reduced agreement {agr:.6f} max err {err:.3e}")


@pytest.mark.parametrize("flags", FLAG_SETS)
@pytest.mark.parametrize("integer", [True, False], ids=["int", "normal"])
def test_c4_shape_reduced(flags, integer):
    w = synth.scaled(synth.C4, q_len=8192 + 70, kv_len=8192 + 70, n_q_heads=4, n_kv_heads=2, integer=integer)
    nqb = w.n_query_blocks
    units = [(0, h, qb) for h in range(w.n_q_heads) for qb in (0, 15, 16, 17, 40, 64, 65, nqb - 2, nqb - 1)]
    U.run_case(w, flags, units=units)


@pytest.mark.parametrize("flags", FLAG_SETS)
@pytest.mark.parametrize("integer", [True, False], ids=["int", "normal"])
def test_decode_contiguous(flags, integer):
    w = synth.scaled(synth.C3, batch=3, kv_len=20000, integer=integer)
    U.run_case(w, flags)


@pytest.mark.parametrize("flags", FLAG_SETS)
@pytest.mark.parametrize("integer", [True, False], ids=["int", "normal"])
def test_decode_ragged_paged(flags, integer):
    w = synth.scaled(synth.C5, batch=6, kv_len=9000, ragged=(700, 9000), integer=integer)
    U.run_case(w, flags)


@pytest.mark.parametrize("flags", FLAG_SETS)
@pytest.mark.parametrize("integer", [True, False], ids=["int", "normal"])
def test_prefill_paged(flags, integer):
    # causal prefill over a paged KV pool (16-token pages, random page table), two sequences
    w = synth.scaled(synth.C2, batch=2, q_len=3000, kv_len=3000, n_q_heads=4, n_kv_heads=2, k=256, spike_every=512,
                     page_size=16, integer=integer)
    nqb = w.n_query_blocks
    units = [(b, h, qb) for b in range(2) for h in range(4) for qb in (0, 3, 4, 5, 20, 50, nqb - 2, nqb - 1)]
    U.run_case(w, flags, units=units)


@pytest.mark.parametrize("flags", FLAG_SETS)
@pytest.mark.parametrize("q_len,bq", [(32, 32), (100, 32), (64, 64), (7, 4)])
def test_chunk_of_queries_over_long_context(flags, q_len, bq):
    # q_len < kv_len: the last q_len positions of each sequence are queried (chunked prefill, or decode
    # with several query rows per sequence as in speculative decoding); ragged lengths
    for integer in (True, False):
        w = synth.Workload("chunk", 3, 8, 2, 128, q_len, 5000, 256, bq, 2, "bf16", rho=0.9, ragged=(600, 5000),
                           integer=integer, seed=55)
        U.run_case(w, flags)


@pytest.mark.parametrize("integer", [True, False], ids=["int", "normal"])
def test_decode_large_batch(integer):
    # more than 8192 (sequence, head) problems select the wave-per-problem decode kernels (a workgroup per problem
    # below that)
    w = synth.scaled(synth.C5, batch=288, kv_len=3000, ragged=(600, 3000), integer=integer)
    rng = np.random.default_rng(2)
    units = [(int(b), int(h), 0) for b, h in zip(rng.integers(0, 288, 300), rng.integers(0, 32, 300))]
    U.run_case(w, 0, units=sorted(set(units)))


@pytest.mark.parametrize("bk,d,k,page,T", [(1, 128, 64, 0, 1500), (2, 128, 512, 16, 1500), (1, 64, 512, 0, 1500), (4, 128, 1024, 64, 2500),
                                           (8, 128, 2048, 0, 3000), (2, 64, 2048, 0, 2500)])
def test_decode_wave_per_problem_variants(bk, d, k, page, T):
    # the wave-per-problem kernels (more than 8192 problems) at every block width, both head dims, k/bk from 64 to
    # 1024, contiguous and paged, ragged: 8320 problems of 8 query heads over one kv head, sampled against the oracle
    w = synth.Workload("decode_wpp", 1040, 8, 1, d, 1, T, k, 1, bk, "bf16", rho=0.9, ragged=(T // 5, T), page_size=page,
                       integer=True, seed=93)
    rng = np.random.default_rng(bk * 100 + d)
    units = sorted({(int(b), int(h), 0) for b, h in zip(rng.integers(0, 1040, 250), rng.integers(0, 8, 250))} | {(0, 0, 0), (1039, 7, 0)})
    U.run_case(w, 0, units=units)


@pytest.mark.parametrize("bk,d,k,hq,hkv", [(1, 128, 64, 4, 4), (4, 128, 1024, 8, 2), (2, 64, 256, 6, 2), (1, 64, 512, 4, 1),
                                          (4, 64, 2048, 2, 1)])
def test_decode_variants(bk, d, k, hq, hkv):
    # block sizes, head dims, group sizes and k/bk (64 .. 512) the decode kernels are instantiated for
    for integer in (True, False):
        w = synth.Workload("decode_var", 5, hq, hkv, d, 1, 12000, k, 1, bk, "bf16", rho=0.9, ragged=(300, 12000),
                           page_size=16 if bk == 4 else 0, integer=integer, seed=91)
        U.run_case(w, 0)


@pytest.mark.parametrize("flags", FLAG_SETS)
@pytest.mark.parametrize("T,k,bq,bk,d,hq,hkv,dtype", [
    (1, 8, 1, 1, 64, 1, 1, "fp32"),        # a single token
    (37, 64, 4, 2, 64, 2, 1, "fp32"),      # k >= T: everything visible is selected (dense)
    (130, 12, 8, 4, 128, 2, 2, "bf16"),    # kb = 3, not a power of two; T % bk != 0; short last block
    (257, 10, 1, 1, 64, 1, 1, "bf16"),     # token-level search (bq = bk = 1), kb = 10
    (300, 64, 64, 16, 128, 4, 1, "fp32"),  # largest blocks
    (1500, 2048, 16, 2, 64, 1, 1, "bf16"), # kb = 1024 (the maximum), mostly dense
    (5000, 2048, 16, 2, 64, 1, 1, "fp32"), # kb = 1024 with pruning
])
def test_edge_shapes(flags, T, k, bq, bk, d, hq, hkv, dtype):
    for integer in (True, False):
        w = synth.Workload("edge", 2, hq, hkv, d, T, T, k, bq, bk, dtype, rho=0.9, integer=integer, seed=77)
        units = None
        if T >= 1500:
            nqb = w.n_query_blocks
            units = [(b, 0, qb) for b in range(2) for qb in (0, nqb // 2, nqb - 1)]
        U.run_case(w, flags, units=units)


def test_empty_batch_and_strided_views():
    import paper_2406_09827_amd as hipattn
    w = synth.scaled(synth.C1, integer=True, n_q_heads=2)
    x = synth.make_inputs(w, device="cuda", threads=1)
    # zero sequences: nothing is launched, nothing is written
    q0 = x["Q"][:0]
    idx0 = hipattn.hip_mask_estimate(q0, x["K"][:0], w.k, w.bq, w.bk)
    assert idx0.numel() == 0
    # token-major storage [B, T, H, d] viewed as [B, H, T, d]: strides go through the ABI
    Qt = x["Q"].permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    Kt = x["K"].permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    Vt = x["V"].permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    assert not Qt.is_contiguous()
    a = hipattn.hip_mask_estimate(x["Q"], x["K"], w.k, w.bq, w.bk)
    bidx = hipattn.hip_mask_estimate(Qt, Kt, w.k, w.bq, w.bk)
    assert torch.equal(a, bidx)
    oa = hipattn.hip_sparse_attn(x["Q"], x["K"], x["V"], a, w.k, w.bq, w.bk)
    ob = hipattn.hip_sparse_attn(Qt, Kt, Vt, a, w.k, w.bq, w.bk, out=torch.empty_like(Qt))
    assert torch.equal(oa, ob)


# ---- sink + sliding window in the sparse attention, mask reuse across decode steps -------------

@pytest.mark.parametrize("flags", FLAG_SETS)
@pytest.mark.parametrize("n_sink,n_window", [(4, 64), (128, 16), (0, 100), (33, 0), (5000, 7)])
def test_prefill_sink_window(flags, n_sink, n_window):
    w = synth.scaled(synth.C2, q_len=3000 + 17, kv_len=3000 + 17, n_q_heads=4, n_kv_heads=2, k=256, spike_every=1024)
    nqb = w.n_query_blocks
    units = [(0, h, qb) for h in range(4) for qb in (0, 1, 2, 3, 4, 5, 9, 40, nqb - 2, nqb - 1)]
    U.run_case(w, flags, units=units, n_sink=n_sink, n_window=n_window)


@pytest.mark.parametrize("flags", FLAG_SETS)
def test_prefill_sink_window_fp32_and_big_blocks(flags):
    U.run_case(synth.C1, flags, n_sink=8, n_window=48)
    w = synth.scaled(synth.C4, q_len=4096 + 70, kv_len=4096 + 70, n_q_heads=2, n_kv_heads=1, k=512)
    nqb = w.n_query_blocks
    U.run_case(w, flags, units=[(0, h, qb) for h in range(2) for qb in (0, 1, 2, 7, 30, nqb - 1)], n_sink=16, n_window=200)


@pytest.mark.parametrize("flags", FLAG_SETS)
@pytest.mark.parametrize("n_sink,n_window", [(4, 64), (300, 5), (0, 1), (9, 0)])
def test_decode_sink_window(flags, n_sink, n_window):
    w = synth.scaled(synth.C5, batch=5, kv_len=7000, ragged=(100, 7000))
    U.run_case(w, flags, n_sink=n_sink, n_window=n_window)
    w = synth.scaled(synth.C3, batch=2, kv_len=9000)
    U.run_case(w, flags, n_sink=n_sink, n_window=n_window)


def test_mask_reuse_across_decode_steps():
    """Alg. 2 with a refresh period: the mask of step 0 serves the next steps; the sliding window
    covers the tokens appended since.  Each step is checked against the oracle on the same indices."""
    import oracle
    import paper_2406_09827_amd as hipattn
    r_m, n_window, n_sink = 8, 16, 4
    w = synth.scaled(synth.C3, batch=3, kv_len=6000 + r_m)
    x = synth.make_inputs(w, device="cuda", threads=2)
    lens0 = torch.tensor([6000, 3500, 811], dtype=torch.int32, device="cuda")
    hx = U.host(x)
    idx = None
    for step in range(r_m):
        lens = (lens0 + step).contiguous()
        if step == 0:
            idx = hipattn.hip_mask_estimate(x["Q"], x["K"], w.k, 1, w.bk, kv_lens=lens)
        out = hipattn.hip_sparse_attn(x["Q"], x["K"], x["V"], idx, w.k, 1, w.bk, kv_lens=lens, n_sink=n_sink, n_window=n_window)
        p = oracle.Problem(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, 1, w.kv_len, w.k, 1, w.bk,
                           kv_lens=lens.cpu().numpy(), n_sink=n_sink, n_window=n_window, n_threads=8)
        ref = oracle.sparse_attn(p, hx["Q"], hx["K"], hx["V"], idx.cpu().numpy())
        U.check_output(out.float().cpu().numpy(), ref, "bf16")


# ---- scoring variants of the mask estimation: sampling strides and representative position ------

@pytest.mark.parametrize("flags", FLAG_SETS)
@pytest.mark.parametrize("bq,bk,b_sq,b_sk,rep_pos", [(32, 2, 2, 2, 0), (64, 4, 2, 1, 0), (32, 8, 1, 2, 1), (32, 4, 4, 4, 2),
                                                     (16, 2, 1, 1, 1), (48, 2, 2, 1, 2)])
def test_prefill_scoring_variants(flags, bq, bk, b_sq, b_sk, rep_pos):
    for integer in (True, False):
        w = synth.Workload("variants", 1, 4, 2, 128, 2500, 2500, 64 * bk, bq, bk, "bf16", rho=0.95, spike_every=512,
                           integer=integer, seed=66)
        nqb = w.n_query_blocks
        units = [(0, h, qb) for h in range(4) for qb in sorted({0, 3, 4, 5, 9, nqb // 2, nqb - 2, nqb - 1})]
        U.run_case(w, flags, units=units, b_sq=b_sq, b_sk=b_sk, rep_pos=rep_pos)


@pytest.mark.parametrize("top_r", [1, 16, 40, 127])
def test_top_r_channels(top_r):
    # scores over each query row's top_r strongest channels: prefill (bf16, d = 128), decode (ragged, paged) and fp32 d = 64
    for integer in (True, False):
        w = synth.Workload("variants_topr", 1, 4, 2, 128, 1500, 1500, 128, 32, 2, "bf16", rho=0.95, spike_every=512,
                           integer=integer, seed=68)
        nqb = w.n_query_blocks
        U.run_case(w, 0, units=[(0, h, qb) for h in range(4) for qb in sorted({0, 3, 5, nqb // 2, nqb - 1})], top_r=top_r)
        w = synth.Workload("variants_topr_dec", 4, 4, 2, 128, 1, 6000, 256, 1, 2, "bf16", rho=0.9, ragged=(300, 6000),
                           page_size=16, integer=integer, seed=69)
        U.run_case(w, 0, top_r=top_r)
    U.run_case(synth.C1_INT, 0, top_r=min(top_r, 63))
    U.run_case(synth.C1, 0, top_r=min(top_r, 63), b_sq=2, rep_pos=2)


def test_fp32_scoring_variants():
    U.run_case(synth.C1_INT, 0, b_sq=4, b_sk=2, rep_pos=2)
    U.run_case(synth.C1, 0, b_sq=2, b_sk=1, rep_pos=1)


@pytest.mark.parametrize("flags", FLAG_SETS)
@pytest.mark.parametrize("bk,b_sk,rep_pos,paged", [(2, 2, 0, False), (4, 2, 1, True), (8, 2, 2, False), (4, 4, 0, True), (2, 1, 2, True)])
def test_decode_scoring_variants(flags, bk, b_sk, rep_pos, paged):
    for integer in (True, False):
        w = synth.Workload("variants_dec", 6, 8, 2, 128, 1, 9000, 128 * bk, 1, bk, "bf16", rho=0.9, ragged=(300, 9000),
                           page_size=16 if paged else 0, integer=integer, seed=67)
        U.run_case(w, flags, b_sk=b_sk, rep_pos=rep_pos)


def test_measurement_probes():
    # the copy probe moves every byte; the MFMA probe runs and writes finite sums
    from paper_2406_09827_amd import probes as hipattn
    src = torch.randint(0, 255, (3 * 1024 * 1024 + 16,), dtype=torch.uint8, device="cuda")
    dst = torch.zeros_like(src)
    hipattn.probe_copy(dst, src)
    assert torch.equal(dst, src)
    red = torch.zeros(hipattn.PROBE_READ_WORDS, dtype=torch.int32, device="cuda")
    hipattn.probe_read(red, src)
    words = src[:src.numel() // 4 * 4].view(torch.int32)
    fold = lambda t: int(np.bitwise_xor.reduce(t.cpu().numpy().view(np.uint32)))
    assert fold(red) == fold(words)
    out = torch.full((8 * 256,), float("nan"), device="cuda")
    assert hipattn.probe_mfma(out, 8, 16) == 8 * 4 * 16 * 4 * 2.0 * 32 * 32 * 16
    torch.cuda.synchronize()
    assert torch.isfinite(out).all()
    # the gather probe reads inside its buffer for every slice count and run length (it is checked by what it
    # returns only: its reads leave no trace but the time they take)
    buf = torch.zeros(8 << 20, dtype=torch.uint8, device="cuda")
    words = torch.full((64 * 256,), 1, dtype=torch.int32, device="cuda")
    for slices, run in ((1, 1), (8, 2), (8, 32), (3, 4)):
        assert hipattn.probe_gather(words, buf, slices, run, 64, 8) == 64 * 4 * 8 * 8192
    torch.cuda.synchronize()
    assert int(words.abs().sum()) == 0       # XOR of zeros


# ---- seeded sweep over shapes and options (integer-valued inputs: indices must match bit for bit) ----

def _sweep_case(seed):
    rng = np.random.default_rng(1000 + seed)
    d = int(rng.choice([64, 128]))
    hkv = int(rng.choice([1, 2, 3]))
    g = int(rng.choice([1, 2, 4]))
    bk = int(rng.choice([1, 2, 4, 8, 16]))
    decode = bool(rng.integers(0, 2))
    dtype = "bf16" if rng.integers(0, 4) else "fp32"
    kb = int(rng.choice([1, 3, 8, 32, 64, 100, 256]))
    paged = bool(rng.integers(0, 2))
    page = int(rng.choice([bk, 2 * bk, 4 * bk, 16 * bk])) if paged else 0
    if decode:
        B, bq, q_len = int(rng.integers(1, 6)), 1, 1
        T = int(rng.integers(1, 6000))
        ragged = (max(1, T // 7), T) if rng.integers(0, 2) else None
    else:
        B = int(rng.integers(1, 3))
        bq = int(rng.choice([1, 4, 16, 32, 48, 64]))
        T = int(rng.integers(bq, 1800))
        q_len = T if rng.integers(0, 3) else int(rng.integers(1, T + 1))   # sometimes a chunk of rows at the end
        ragged = None
    b_sk = int(rng.choice([x for x in (1, 2, 4) if bk % x == 0]))
    b_sq = int(rng.choice([x for x in (1, 2, 4) if x <= bq]))
    opts = dict(b_sq=b_sq, b_sk=b_sk, rep_pos=int(rng.integers(0, 3)),
                n_sink=int(rng.choice([0, 0, 3, 16])), n_window=int(rng.choice([0, 0, 5, 64])),
                top_r=int(rng.choice([0, 0, 0, 5, d // 2])), sm_scale=float(rng.choice([0.0, 0.0, 0.03, 0.4, 1.5])))
    w = synth.Workload(f"sweep{seed}", B, hkv * g, hkv, d, q_len, T, kb * bk, bq, bk, dtype, rho=0.9, ragged=ragged,
                       page_size=page, integer=True, seed=4000 + seed)
    return w, opts


@pytest.mark.parametrize("seed", range(500))
def test_seeded_shape_sweep(seed):
    w, opts = _sweep_case(seed)
    print(w, opts, flush=True)
    units = None
    if w.n_query_blocks * w.batch * w.n_q_heads > 400:
        rng = np.random.default_rng(seed)
        nqb = w.n_query_blocks
        units = sorted({(int(rng.integers(0, w.batch)), int(rng.integers(0, w.n_q_heads)), int(q))
                        for q in list(rng.integers(0, nqb, 60)) + [0, nqb - 1]})
    U.run_case(w, 0, units=units, **opts)


@pytest.mark.parametrize("sm_scale", [0.5, 0.01])
def test_softmax_scale_extremes(sm_scale):
    # a scale that makes the softmax nearly one-hot (running maximum jumps by far more than the lazy-rescale
    # slack) and one that makes it nearly uniform; prefill and decode
    w = synth.scaled(synth.C2, q_len=3000, kv_len=3000, n_q_heads=4, n_kv_heads=2, spike_every=700)
    nqb = w.n_query_blocks
    U.run_case(w, 0, units=[(0, h, qb) for h in range(4) for qb in (0, 5, 20, nqb // 2, nqb - 1)], sm_scale=sm_scale)
    U.run_case(synth.scaled(synth.C3, batch=3, kv_len=9000), 0, sm_scale=sm_scale)
    U.run_case(synth.scaled(synth.C5, batch=5, kv_len=7000, ragged=(400, 7000)), 0, sm_scale=sm_scale, n_sink=4, n_window=32)


def test_decode_step_replayed_from_a_graph():
    # mask estimation + sparse attention captured once into a HIP graph and replayed with eager work and
    # synchronisations in between: every replay must reproduce the eager result bit for bit (the calls
    # allocate nothing and record no memset nodes, so a serving loop can capture them)
    import paper_2406_09827_amd as hipattn
    w = synth.scaled(synth.C5, batch=8, kv_len=5000, ragged=(600, 5000))
    x = synth.make_inputs(w, device="cuda", threads=4)
    idx = torch.empty((w.batch, w.n_q_heads, 1, w.kb), dtype=torch.int32, device="cuda")
    out = torch.empty_like(x["Q"])

    def step():
        hipattn.hip_mask_estimate(x["Q"], x["K"], w.k, w.bq, w.bk, kv_lens=x["kv_lens"], page_table=x["page_table"],
                                  indices=idx)
        hipattn.hip_sparse_attn(x["Q"], x["K"], x["V"], idx, w.k, w.bq, w.bk, kv_lens=x["kv_lens"],
                                page_table=x["page_table"], out=out, n_sink=4, n_window=16)

    step()
    torch.cuda.synchronize()
    idx_ref, out_ref = idx.clone(), out.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()                                  # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    for r in range(3):
        idx.fill_(-7)
        out.zero_()
        x["Q"].mul_(1.0)                        # unrelated eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(idx, idx_ref), f"replay {r}: indices differ"
        assert torch.equal(out, out_ref), f"replay {r}: output differs"


@pytest.mark.parametrize("rep_pos", [1, 2])
def test_c4_and_c2_shapes_with_first_and_last_representative(rep_pos):
    # the list rounds of the prefill kernel (scores carried from parent to child) at the benchmark shapes:
    # k/bk = 512 with 64-row query blocks, k/bk = 256 with 32-row blocks; and the decode carry variant at k/bk = 512
    w = synth.scaled(synth.C4, q_len=8192 + 70, kv_len=8192 + 70, n_q_heads=4, n_kv_heads=2, integer=True)
    nqb = w.n_query_blocks
    U.run_case(w, 0, units=[(0, h, qb) for h in range(4) for qb in (0, 15, 16, 17, 40, 64, 65, nqb - 2, nqb - 1)], rep_pos=rep_pos)
    w = synth.scaled(synth.C2, q_len=4096 + 40, kv_len=4096 + 40, n_q_heads=8, n_kv_heads=2, spike_every=1024)
    nqb = w.n_query_blocks
    U.run_case(w, 0, units=[(0, h, qb) for h in range(8) for qb in (0, 8, 9, 17, 33, 64, nqb - 2, nqb - 1)], rep_pos=rep_pos)
    w = synth.Workload("dec_kb512", 3, 8, 2, 128, 1, 40000, 2048, 1, 4, "bf16", rho=0.9, ragged=(5000, 40000), integer=True, seed=93)
    U.run_case(w, 0, rep_pos=rep_pos)


def test_plain_c_caller_of_the_abi():
    # tests/c_abi/c_abi_smoke.c: a C program that links the library, no Python in the call path
    import os
    import subprocess
    exe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_abi", "c_abi_smoke")
    assert os.path.exists(exe), "not built: run __graft_entry__.build()"
    r = subprocess.run([exe], capture_output=True, text=True, timeout=100)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "ok" in r.stdout


def test_rows_four_gigabytes_apart_in_total():
    # K and V as views whose (sequence, head) slice spans 4 GiB (1024 rows, 4 MiB row pitch): the tuned kernels
    # switch from 32-bit lane offsets to 64-bit row addresses (attention) resp. to the generic kernel (mask);
    # results must equal those on the packed tensors
    import paper_2406_09827_amd as hipattn
    w = synth.Workload("wide", 1, 2, 1, 128, 1024, 1024, 64, 32, 2, "bf16", rho=0.9, integer=True, seed=95)
    x = synth.make_inputs(w, device="cuda", threads=1)
    pitch = 1 << 21  # elements
    views = {}
    for name in ("K", "V"):
        big = torch.empty(w.kv_len * pitch, dtype=torch.bfloat16, device="cuda")
        v = big.as_strided((1, 1, w.kv_len, w.head_dim), (w.kv_len * pitch, w.kv_len * pitch, pitch, 1))
        v.copy_(x[name])
        views[name] = v
    a = hipattn.hip_mask_estimate(x["Q"], x["K"], w.k, w.bq, w.bk)
    b = hipattn.hip_mask_estimate(x["Q"], views["K"], w.k, w.bq, w.bk)
    assert torch.equal(a, b)
    oa = hipattn.hip_sparse_attn(x["Q"], x["K"], x["V"], a, w.k, w.bq, w.bk)
    ob = hipattn.hip_sparse_attn(x["Q"], views["K"], views["V"], a, w.k, w.bq, w.bk)
    torch.cuda.synchronize()
    assert torch.equal(oa, ob)
    del views
    torch.cuda.empty_cache()


def test_single_query_row_with_a_prefill_block_size():
    # q_len = 1 with bq = 32: the row is its own query block (same result as bq = 1); served by the decode kernels
    import paper_2406_09827_amd as hipattn
    w1 = synth.Workload("one_row_bq1", 3, 4, 2, 128, 1, 5000, 128, 1, 2, "bf16", rho=0.9, ragged=(900, 5000), integer=True, seed=96)
    w32 = synth.scaled(w1, bq=32)
    x = synth.make_inputs(w1, device="cuda", threads=1)
    a = hipattn.hip_mask_estimate(x["Q"], x["K"], w1.k, 1, w1.bk, kv_lens=x["kv_lens"], max_kv_len=w1.kv_len)
    b = hipattn.hip_mask_estimate(x["Q"], x["K"], w32.k, 32, w32.bk, kv_lens=x["kv_lens"], max_kv_len=w32.kv_len, b_sq=2)
    assert torch.equal(a, b)
    U.run_case(w32, 0, b_sq=2, n_window=8)


def test_seeded_shape_sweep_real_valued():
    # the same sweep on real-valued inputs: every case must give valid indices and an output within tolerance of
    # the oracle's on those indices; index agreement is judged over all cases together (a single near-tie can
    # flip one entry of a tiny case), and no case may fall below 90 %
    total = 0.0
    n = 0
    for seed in range(150):
        w, opts = _sweep_case(seed)
        w = synth.scaled(w, integer=False, rho=0.9)
        # (softmax scales of 0.4 and 1.5 are part of the sweep: the logits of these unnormalised keys then reach
        # +-75; the fp32 bound follows the logit and value sizes, see tests/gpu_util.py)
        units = None
        if w.n_query_blocks * w.batch * w.n_q_heads > 400:
            rng = np.random.default_rng(seed)
            nqb = w.n_query_blocks
            units = sorted({(int(rng.integers(0, w.batch)), int(rng.integers(0, w.n_q_heads)), int(q))
                            for q in list(rng.integers(0, nqb, 60)) + [0, nqb - 1]})
        print(seed, w, opts, flush=True)
        agr, _ = U.run_case(w, 0, units=units, min_agreement=0.9, **opts)
        total += agr
        n += 1
    assert total / n >= 0.999, f"mean agreement {total / n:.5f}"
    print(f"bf16 outputs of |ref| >= 4: {U.FULL_ULP_COUNT[1]} of {U.FULL_ULP_COUNT[0]} a full unit in the last place away")


@pytest.mark.parametrize("integer", [True, False], ids=["int", "normal"])
def test_k_over_bk_up_to_1024(integer):
    # k/bk = 1024 (the maximum) and 768 on the tuned kernels: prefill with 32- and 64-row query blocks, decode
    # contiguous and paged, last-block representative
    w = synth.Workload("kb1024", 1, 4, 2, 128, 20000 + 30, 20000 + 30, 2048, 32, 2, "bf16", rho=0.95, spike_every=4096,
                       integer=integer, seed=97)
    nqb = w.n_query_blocks
    U.run_case(w, 0, units=[(0, h, qb) for h in range(4) for qb in (0, 31, 32, 33, 70, nqb // 2, nqb - 2, nqb - 1)])
    w = synth.Workload("kb768", 1, 2, 1, 64, 30000, 30000, 3072, 64, 4, "bf16", rho=0.95, integer=integer, seed=98)
    nqb = w.n_query_blocks
    U.run_case(w, 0, units=[(0, h, qb) for h in range(2) for qb in (0, 47, 48, 49, 100, nqb - 1)], rep_pos=2)
    w = synth.Workload("kb1024_dec", 3, 4, 2, 128, 1, 50000, 2048, 1, 2, "bf16", rho=0.9, ragged=(3000, 50000),
                       integer=integer, seed=99)
    U.run_case(w, 0)
    w = synth.Workload("kb1024_dec_paged", 2, 4, 1, 64, 1, 40000, 4096, 1, 4, "bf16", rho=0.9, ragged=(9000, 40000), page_size=64,
                       integer=integer, seed=100)
    U.run_case(w, 0, rep_pos=1)


@pytest.mark.parametrize("integer", [True, False], ids=["int", "normal"])
def test_paged_prefill_variants(integer):
    # prefill over a paged pool on every tuned mask kernel: k/bk = 256 (page ids kept per branch slot), 512 with 32-row
    # (packed list rounds) and 64-row query blocks, 1024 (page look-ups issued from the tile loop), list rounds with the
    # first / last representative, a chunk of rows at the end of a long context (one work item per workgroup), and a
    # page size that is not a power of two (generic kernel)
    w = synth.Workload("paged_pf", 2, 4, 2, 128, 9000 + 30, 9000 + 30, 512, 32, 2, "bf16", rho=0.95, spike_every=2048,
                       page_size=64, integer=integer, seed=111)
    nqb = w.n_query_blocks
    units = [(b, h, qb) for b in range(2) for h in range(4) for qb in (0, 15, 16, 17, 70, nqb // 2, nqb - 2, nqb - 1)]
    for rep_pos in (0, 1, 2):
        U.run_case(w, 0, units=units, rep_pos=rep_pos)
    U.run_case(synth.scaled(w, k=1024, page_size=16), 0, units=units, n_sink=4, n_window=33)
    U.run_case(synth.scaled(w, k=1024, bq=64, page_size=256), 0, units=[u for u in units if u[2] < nqb // 2], b_sq=2)
    U.run_case(synth.scaled(w, k=2048, page_size=128), 0, units=units, rep_pos=2)
    U.run_case(synth.scaled(w, k=2048, head_dim=64, bk=4, page_size=32), 0, units=units, b_sk=2)
    U.run_case(synth.scaled(w, q_len=64, page_size=8), 0)
    U.run_case(synth.scaled(w, q_len=64, k=1024, page_size=8), 0, rep_pos=2)
    U.run_case(synth.scaled(w, q_len=96, k=1024, bq=64, page_size=8, head_dim=64), 0, rep_pos=1)
    # four query heads per kv head: the four work items of a workgroup share a sequence, which the variant with the page
    # table cached in LDS needs; with 8-key pages the table (1129 pages) is too long for it
    w4 = synth.scaled(w, n_q_heads=8, n_kv_heads=2)
    units4 = [(b, h, qb) for b in range(2) for h in (0, 3, 4, 7) for qb in (0, 15, 16, 70, nqb // 2, nqb - 1)]
    for rep_pos in (0, 2):
        U.run_case(w4, 0, units=units4, rep_pos=rep_pos, n_window=9)
    U.run_case(synth.scaled(w4, page_size=8), 0, units=units4)
    U.run_case(synth.scaled(w4, head_dim=64, page_size=16, bk=4, k=1024), 0, units=units4, b_sk=2)
    U.run_case(synth.scaled(w, page_size=48), 0, units=units)
    U.run_case(synth.scaled(w, page_size=6, batch=1), 0, units=[u for u in units if u[0] == 0], rep_pos=2)


@pytest.mark.parametrize("flags", FLAG_SETS)
@pytest.mark.parametrize("resident_frac", [0.0, 0.5, 1.0])
def test_token_bank_decode(flags, resident_frac):
    # the paper's offloading layout (Sec. 3.3): a bank of resident pages, misses read from a backing pool, the map of
    # pages read.  Ragged paged decode on the tuned and the generic kernels; a block per page and larger pages.
    w = synth.Workload("bank_dec", 5, 8, 2, 128, 1, 7000, 256, 1, 2, "bf16", rho=0.9, ragged=(900, 7000), page_size=16,
                       integer=True, seed=121)
    miss = U.run_bank_case(w, resident_frac, flags, n_sink=3, n_window=20)
    assert abs(miss - (1.0 - resident_frac)) < 0.1
    U.run_bank_case(synth.scaled(w, page_size=2, head_dim=64), resident_frac, flags)
    U.run_bank_case(synth.scaled(w, bk=4, k=512, page_size=64, batch=2), resident_frac, flags, rep_pos=2, b_sk=2)
    U.run_bank_case(synth.scaled(w, batch=300, n_q_heads=2, n_kv_heads=1, kv_len=2000, ragged=(300, 2000), k=128),
                    resident_frac, flags)   # wave-per-problem variants


@pytest.mark.parametrize("flags", FLAG_SETS)
def test_token_bank_prefill(flags):
    # the same over the prefill kernels: 32- and 64-row query blocks, list rounds, k/bk = 512 and 1024, a chunk of rows
    w = synth.Workload("bank_pf", 2, 4, 2, 128, 2500 + 30, 2500 + 30, 128, 32, 2, "bf16", rho=0.95, page_size=32,
                       integer=True, seed=122)
    U.run_bank_case(w, 0.5, flags, n_sink=4, n_window=40)
    U.run_bank_case(synth.scaled(w, bq=64, head_dim=64, page_size=8), 0.3, flags, rep_pos=1)
    U.run_bank_case(synth.scaled(w, q_len=70), 0.7, flags, rep_pos=2)
    if not flags:
        U.run_bank_case(synth.scaled(w, k=1024, q_len=400, batch=1, kv_len=6000), 0.5)
        U.run_bank_case(synth.scaled(w, k=2048, q_len=200, batch=1, kv_len=6000, page_size=4), 0.5)
    U.run_bank_case(synth.scaled(w, dtype="fp32", q_len=300, head_dim=64), 0.5, flags)
    U.run_bank_case(synth.scaled(w, page_size=6, q_len=300), 0.5, flags)   # not a power of two


def test_pages_read_map_accumulates():
    # the library only ever stores 1 into the map: bytes set before the call stay set, two calls leave the union
    w = synth.Workload("bank_acc", 2, 4, 2, 128, 1, 4000, 128, 1, 2, "bf16", rho=0.9, ragged=(2000, 4000), page_size=16,
                       integer=True, seed=124)
    x = synth.make_inputs(w, device="cuda", threads=4)
    kw = dict(kv_lens=x["kv_lens"], page_table=x["page_table"])
    a = torch.zeros_like(x["page_table"], dtype=torch.uint8)
    b = torch.zeros_like(a)
    idx = hipattn.hip_mask_estimate(x["Q"], x["K"], w.k, w.bq, w.bk, touched=a, **kw)
    hipattn.hip_sparse_attn(x["Q"], x["K"], x["V"], idx, w.k, w.bq, w.bk, touched=b, n_window=5, **kw)
    both = a.clone()
    both[0, -1] = 1                                   # a byte of the caller's (beyond the first sequence's pages)
    hipattn.hip_sparse_attn(x["Q"], x["K"], x["V"], idx, w.k, w.bq, w.bk, touched=both, n_window=5, **kw)
    torch.cuda.synchronize()
    want = a | b
    want[0, -1] = 1
    assert torch.equal(both, want) and bool(a.any()) and bool(b.any()) and int(a.max()) == 1


def test_token_bank_in_host_memory():
    # the backing pool in pinned host memory (an offloaded KV cache): misses are read over the host link
    w = synth.Workload("bank_host", 4, 8, 2, 128, 1, 5000, 256, 1, 2, "bf16", rho=0.9, ragged=(900, 5000), page_size=16,
                       integer=True, seed=123)
    U.run_bank_case(w, 0.8, host_backing=True, n_window=16)
    U.run_bank_case(synth.scaled(w, q_len=64, bq=32, batch=1, ragged=None), 0.8, host_backing=True)


@pytest.mark.parametrize("integer", [True, False], ids=["int", "normal"])
def test_direct_to_lds_variant_limits(integer):
    # the mask kernel with direct-to-LDS loads serves contiguous K of up to 32 MB per kv head (128k keys at head dim
    # 128): the largest context it takes, the first one it leaves to the register-staged kernel, 64k keys, a short last
    # key block, list rounds (first / last representative), key sampling and a ragged batch
    w = synth.Workload("direct_128k", 1, 4, 1, 128, 8192, 131072, 512, 32, 2, "bf16", rho=0.95, spike_every=8192,
                       integer=integer, seed=131)
    nqb = w.n_query_blocks
    units = [(0, h, qb) for h in range(4) for qb in (0, 1, 77, nqb // 2, nqb - 2, nqb - 1)]
    U.run_case(w, 0, units=units)
    U.run_case(synth.scaled(w, kv_len=131072 + 64), 0, units=units)
    U.run_case(synth.scaled(w, kv_len=65536 + 64), 0, units=units)
    U.run_case(synth.scaled(w, kv_len=40001, q_len=9001), 0, units=[(0, h, qb) for h in range(4) for qb in (0, 100, 281)], rep_pos=2)
    U.run_case(synth.scaled(w, kv_len=30000, q_len=30000, bk=4, k=1024), 0,
               units=[(0, h, qb) for h in range(4) for qb in (0, 31, 32, 33, 500, 937)], rep_pos=1, b_sk=2, n_window=17)
    wr = synth.Workload("direct_ragged", 3, 4, 2, 128, 3000, 9000, 256, 32, 2, "bf16", rho=0.9, ragged=(3500, 9000),
                        integer=integer, seed=132)
    nqb = wr.n_query_blocks
    U.run_case(wr, 0, units=[(b, h, qb) for b in range(3) for h in range(4) for qb in (0, 40, nqb - 1)])


@pytest.mark.parametrize("integer", [True, False], ids=["int", "normal"])
def test_blocks_of_8_and_16_keys(integer):
    # bk = 8 (8 scored rows per block) and bk = 16 with b_sk = 2 on the tuned kernels: prefill at head dim 128,
    # decode (mask with 8 rows per block; attention walks the blocks as pieces of 4 rows)
    w = synth.Workload("bk8", 1, 4, 2, 128, 6000 + 50, 6000 + 50, 1024, 32, 8, "bf16", rho=0.95, spike_every=1024,
                       integer=integer, seed=101)
    nqb = w.n_query_blocks
    units = [(0, h, qb) for h in range(4) for qb in (0, 31, 32, 33, 70, nqb // 2, nqb - 2, nqb - 1)]
    U.run_case(w, 0, units=units)
    U.run_case(synth.scaled(w, bk=16, k=2048, bq=64), 0, units=[(0, h, qb) for h in range(4) for qb in (0, 15, 16, 40, nqb // 2 - 1)],
               b_sk=2, rep_pos=2, n_sink=8, n_window=40)
    wd = synth.Workload("bk8_dec", 4, 4, 2, 128, 1, 30000, 2048, 1, 8, "bf16", rho=0.9, ragged=(3000, 30000),
                        integer=integer, seed=102)
    U.run_case(wd, 0, n_sink=5, n_window=21)
    U.run_case(synth.scaled(wd, bk=16, k=4096, page_size=64, head_dim=64), 0, b_sk=2, rep_pos=1, n_window=50)
    U.run_case(synth.scaled(wd, batch=700, n_q_heads=2, n_kv_heads=1, kv_len=3000, ragged=(400, 3000), k=256), 0)   # wave-per-problem variants


@pytest.mark.parametrize("bk,b_sk,g,rep_pos,b_sq", [(1, 1, 4, 0, 1), (2, 2, 4, 0, 1), (2, 1, 4, 2, 2), (4, 1, 8, 0, 1), (8, 1, 4, 1, 1),
                                                    (2, 1, 8, 0, 1)])
def test_first_round_shared_by_the_heads_of_a_kv_group(bk, b_sk, g, rep_pos, b_sq):
    # more than 512 work items with g a multiple of 4: the four waves of a workgroup are four heads of one query block and
    # go through the first round in step, each tile loaded once (1, 2, 4 and 8 scored rows per block; a ragged last query
    # block; the ensemble's perturbed round, which is the first one for short prefixes).  Against the oracle, and bit for
    # bit against the same call with every head gathering for itself.
    import paper_2406_09827_amd as hipattn
    T = 4500 + 13
    for integer in (True, False):
        w = synth.Workload("shared_round", 1, g, 1, 128, T, T, 96 * bk, 32, bk, "bf16", rho=0.95, spike_every=1024, integer=integer, seed=120 + bk)
        nqb = w.n_query_blocks
        assert g * nqb > 512
        units = [(0, h, qb) for h in range(g) for qb in (3, 4, 7, 12, 40, nqb // 2, nqb - 2, nqb - 1)]
        U.run_case(w, 0, units=units, rep_pos=rep_pos, b_sq=b_sq, b_sk=b_sk)
        x = synth.make_inputs(w, device="cuda", threads=4)
        for ens in (0, 2):
            kw = dict(b_sq=b_sq, b_sk=b_sk, rep_pos=rep_pos, ens_sample=ens, ens_seed=5, ens_r=4.0)
            a = hipattn.hip_mask_estimate(x["Q"], x["K"], w.k, w.bq, w.bk, **kw)
            b = hipattn.hip_mask_estimate(x["Q"], x["K"], w.k, w.bq, w.bk, flags=hipattn.binding.NO_SHARED_ROUND, **kw)
            torch.cuda.synchronize()
            assert torch.equal(a, b)
