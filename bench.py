#!/usr/bin/env python3
"""Benchmark of the HiP hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input that is already
resident in HBM: hip_mask_estimate followed by hip_sparse_attn for one attention layer.
Prints ONE JSON line: the headline metric (`value`: whole-job tokens/s for prefill, us/step for
decode, from wall-clock over the timed steps), per-kernel times from HIP events on the launch stream
(`kernel_ms` mean, `kernel_ms_median`, `kernel_ms_min`), the algorithmic rates of both kernels,
`roofline` for the slower kernel against the roof that binds it (every candidate roof is listed in
`ceilings`; a candidate whose fraction exceeds 1 does not bind and is never chosen), `target_points`
(the default run also times the two points the targets are stated at: C2's shape at T = 131072 and the C3
decode at 128k context) and `cpu_baseline` (the CPU oracle on a bounded sample of the same workload).
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16
# L2 -> compute-unit fill: 16 channels x 128 B per clock per XCD (CDNA3/CDNA4 white papers), 8 XCDs, 2.4 GHz
L2_PEAK_GBS = 16 * 128 * 8 * 2.4


def rounds_of(Tb: int, kb: int) -> int:
    """Rounds a query block with Tb visible key blocks needs: ceil(log2(ceil(Tb/kb)))."""
    if Tb <= kb:
        return 0
    c = -(-Tb // kb)
    return (c - 1).bit_length()


def mask_algorithmic_bytes(w, kv_lens, rep_pos: int = 0) -> float:
    """Key bytes the method has to touch in mask estimation, counted conservatively:
    every round but a unit's last scores 2*kb branches, the last at least kb (nodes that are
    already one block long have a single branch); plus the query block once and the indices.
    With the first or last block as representative, a child that shares its parent's representative
    needs no new bytes: one round of 2*kb branches, kb per later round."""
    size = 2 if w.dtype == "bf16" else 4
    row = w.head_dim * size
    total = 0.0
    for b in range(w.batch):
        kv_len = int(kv_lens[b]) if kv_lens is not None else w.kv_len
        for qb in range(w.n_query_blocks):
            r0 = qb * w.bq
            n = min(w.bq, w.q_len - r0)
            L = min(kv_len, kv_len - w.q_len + r0 + n)
            Tb = -(-L // w.bk) if L > 0 else 0
            R = rounds_of(Tb, w.kb)
            if rep_pos == 0:
                branches = (R - 1) * 2 * w.kb + w.kb if R > 0 else 0
            else:
                branches = (R + 1) * w.kb if R > 0 else 0
            total += branches * w.bk * row + n * row + w.kb * 4
    return total * w.n_q_heads


def attn_algorithmic(w, kv_lens):
    """(flops, bytes) of the sparse attention: 4*rows*keys*d flops per unit over the selected
    keys that exist (k, or the visible prefix when shorter); K and V rows gathered once per unit."""
    size = 2 if w.dtype == "bf16" else 4
    flops = 0.0
    byts = 0.0
    for b in range(w.batch):
        kv_len = int(kv_lens[b]) if kv_lens is not None else w.kv_len
        for qb in range(w.n_query_blocks):
            r0 = qb * w.bq
            n = min(w.bq, w.q_len - r0)
            L = min(kv_len, kv_len - w.q_len + r0 + n)
            keys = min(w.k, max(L, 0))
            flops += 4.0 * n * keys * w.head_dim
            byts += 2.0 * keys * w.head_dim * size + 2.0 * n * w.head_dim * size
    return flops * w.n_q_heads, byts * w.n_q_heads


def mask_score_flops(w, kv_lens, rep_pos: int = 0, b_sq: int = 1, b_sk: int = 1) -> float:
    """Multiply-adds of the block scores as flops: 2 * rows * keys * d per scored branch, with the same
    branch count as mask_algorithmic_bytes."""
    total = 0.0
    for b in range(w.batch):
        kv_len = int(kv_lens[b]) if kv_lens is not None else w.kv_len
        for qb in range(w.n_query_blocks):
            r0 = qb * w.bq
            n = min(w.bq, w.q_len - r0)
            L = min(kv_len, kv_len - w.q_len + r0 + n)
            Tb = -(-L // w.bk) if L > 0 else 0
            R = rounds_of(Tb, w.kb)
            if rep_pos == 0:
                branches = (R - 1) * 2 * w.kb + w.kb if R > 0 else 0
            else:
                branches = (R + 1) * w.kb if R > 0 else 0
            total += 2.0 * branches * (w.bk // b_sk) * -(-n // b_sq) * w.head_dim
    return total * w.n_q_heads


def kernel_source_sha() -> str:
    """Fingerprint of the kernel sources; a counter summary under profiles/ is quoted only while it matches."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2406_09827_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:12]


def read_traffic(name: str):
    """HBM-side bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE) in an EARLIER run,
    kept as a small text file under profiles/ (key = value lines).  Returns (bytes, source) where source says
    which file, when and from which kernel sources it was collected; bytes is None when no file exists or
    when the kernel sources have changed since (a stale counter must not be divided by a fresh time)."""
    rel = os.path.join("profiles", f"traffic_{name}.txt")
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return None, None
    vals = {}
    for line in open(path):
        line = line.split("#")[0]
        if "=" in line:
            k, v = line.split("=", 1)
            vals[k.strip()] = v.strip()
    src = {"file": rel, "collected": vals.get("collected"), "kernel_source_sha": vals.get("kernel_source_sha"),
           "measured_in_this_run": False}
    try:
        byts = float(vals["hbm_bytes_per_launch"])
    except (KeyError, ValueError):
        return None, src
    if vals.get("kernel_source_sha") != kernel_source_sha():
        src["stale"] = True
        return None, src
    return byts, src


def cpu_baseline(w, x, budget_s: float, **variant):
    """The CPU oracle timed on a bounded random sample of (head, query block) units of the same
    workload (mask estimation + sparse attention), all host cores via OpenMP."""
    import numpy as np
    import oracle

    cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "0") or 10**6))
    p = oracle.problem_for(w, x, n_threads=cores, **variant)
    hx = oracle.host_arrays(x)
    rng = np.random.default_rng(1234)
    all_u = oracle.all_units(p)

    def run(n):
        sel = rng.choice(all_u.shape[0], size=min(n, all_u.shape[0]), replace=False)
        units = all_u[sel]
        t0 = time.perf_counter()
        idx = oracle.mask_estimate_units(p, hx["Q"], hx["K"], units)
        oracle.sparse_attn_units(p, hx["Q"], hx["K"], hx["V"], units, idx)
        return time.perf_counter() - t0, units.shape[0]

    t_pilot, n_pilot = run(4 * cores)
    n = int(max(4 * cores, min(all_u.shape[0], n_pilot * budget_s / max(t_pilot, 1e-3))))
    t, n = run(n)
    rows = n * w.bq / w.n_q_heads          # layer-tokens covered by the sample
    if w.q_len < w.kv_len:
        value, unit = t / (n / (w.batch * w.n_q_heads * w.n_query_blocks)) * 1e6, "us/step"
    else:
        value, unit = rows / t, "tokens/s"
    return {"value": value, "unit": unit, "cores": cores, "kind": "oracle",
            "sample": f"{n} random (sequence, head, query block) units of {all_u.shape[0]}, "
                      f"{t:.1f} s wall, extrapolated linearly"}


def _time_ms(fn, reps):
    import torch
    fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    best = float("inf")
    for _ in range(reps):
        a.record()
        fn()
        b.record()
        b.synchronize()
        best = min(best, a.elapsed_time(b))
    return best


def measured_peaks():
    """What this GPU sustains: a 1 GiB device copy (read + write) and back-to-back bf16 MFMAs."""
    import torch
    from paper_2406_09827_amd import probes as hipattn
    src = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    ms_copy = _time_ms(lambda: hipattn.probe_copy(dst, src), 10)
    red = torch.empty(hipattn.PROBE_READ_WORDS, dtype=torch.int32, device="cuda")
    ms_read = _time_ms(lambda: hipattn.probe_read(red, src), 10)
    wgs, iters = 256 * 8, 4096   # 8 workgroups per compute unit, four waves each
    out = torch.empty(wgs * 256, dtype=torch.float32, device="cuda")
    flops = hipattn.probe_mfma(out, wgs, iters)
    ms_mfma = _time_ms(lambda: hipattn.probe_mfma(out, wgs, iters), 5)
    return {"hbm_copy_GB/s": 2 * (1 << 30) / (ms_copy * 1e-3) / 1e9, "hbm_read_GB/s": (1 << 30) / (ms_read * 1e-3) / 1e9, "hbm_published_GB/s": HBM_PEAK_GBS,
            "mfma_bf16_TFLOP/s": flops / (ms_mfma * 1e-3) / 1e12, "mfma_bf16_published_TFLOP/s": MFMA_BF16_PEAK_TFLOPS}


def gather_ceiling(bytes_total: int, run_rows: int):
    """GB/s the gather probe sustains on a buffer of `bytes_total` (capped at 4 GiB) split into 8 slices, one per
    XCD, in runs of `run_rows` rows of 256 bytes: the kernels' access pattern without their arithmetic."""
    import torch
    from paper_2406_09827_amd import probes
    n = int(max(8 << 20, min(bytes_total, 4 << 30))) // (8 * 256) * (8 * 256)
    buf = torch.empty(n, dtype=torch.uint8, device="cuda")
    buf.zero_()
    wgs, tiles = 256 * 8, 64
    out = torch.empty(wgs * 256, dtype=torch.int32, device="cuda")
    run = 1
    while run * 2 <= min(max(run_rows, 1), 32):
        run *= 2
    moved = probes.probe_gather(out, buf, 8, run, wgs, tiles)
    ms = _time_ms(lambda: probes.probe_gather(out, buf, 8, run, wgs, tiles), 5)
    del buf
    return moved / (ms * 1e-3) / 1e9


def dense_yardstick(w, x):
    """torch's dense causal attention on the same Q, K, V (external yardstick only)."""
    import torch
    import torch.nn.functional as F
    g = w.n_q_heads // w.n_kv_heads
    try:
        fn = lambda: F.scaled_dot_product_attention(x["Q"], x["K"], x["V"], is_causal=True, enable_gqa=g > 1)
        ms = _time_ms(fn, 3)
    except Exception as e:  # the yardstick is optional: report why it is missing
        return {"impl": "torch scaled_dot_product_attention", "error": f"{type(e).__name__}: {e}"[:200]}
    flops = 4.0 * w.batch * w.n_q_heads * w.q_len * w.kv_len * w.head_dim / 2
    return {"impl": "torch scaled_dot_product_attention (causal, dense)", "ms": ms, "TFLOP/s": flops / (ms * 1e-3) / 1e12}


def build_workload(args, name=None, seq_len=None):
    from paper_2406_09827_amd import synth
    w = synth.WORKLOADS[name or args.workload]
    seq_len = args.seq_len if seq_len is None else seq_len
    if seq_len > 0:
        w = synth.scaled(w, kv_len=seq_len, q_len=seq_len if w.q_len == w.kv_len else w.q_len,
                         name=f"{w.name}_T{seq_len}")
    if args.q_len > 0:
        w = synth.scaled(w, q_len=args.q_len, name=f"{w.name}_q{args.q_len}")
    if args.page_size >= 0:
        w = synth.scaled(w, page_size=args.page_size, name=f"{w.name}_page{args.page_size}")
    if args.k > 0:
        w = synth.scaled(w, k=args.k, name=f"{w.name}_k{args.k}")
    if args.bk > 0:
        w = synth.scaled(w, bk=args.bk, name=f"{w.name}_bk{args.bk}")
    if args.bq > 0:
        w = synth.scaled(w, bq=args.bq, name=f"{w.name}_bq{args.bq}")
    return w


def pick_roof(cands: dict):
    """The roof that binds = the candidate with the largest fraction that is a fraction (<= 1): a rate above a
    peak means that peak is not what the data passes through (cache hits), so it cannot bound the kernel."""
    valid = {n: c for n, c in cands.items() if c is not None and c["frac"] <= 1.0}
    if not valid:
        return None
    return max(valid, key=lambda n: valid[n]["frac"])


def measure(args, w, tag, steps, warmup, with_cpu):
    """Times `steps` steps of the path on workload `w`; returns the result fields of one JSON line."""
    import torch
    import paper_2406_09827_amd as hipattn
    from paper_2406_09827_amd import synth

    flags = (hipattn.FORCE_GENERIC if args.generic else 0) | (hipattn.binding.NO_SHARED_ROUND if args.no_shared_round else 0)
    t0 = time.perf_counter()
    x = synth.make_inputs(w, device="cuda", threads=16)
    torch.cuda.synchronize()
    print(f"[bench] {w.name}: inputs ready in {time.perf_counter() - t0:.1f} s", file=sys.stderr, flush=True)
    kv_lens = x["kv_lens"].cpu().numpy() if x["kv_lens"] is not None else None
    max_len = None if x["page_table"] is not None else w.kv_len
    x_plain = x   # what the CPU baseline reads
    bank = {}
    if args.resident_frac >= 0:
        if not w.page_size:
            sys.exit("--resident-frac needs a paged workload (c5, or --page-size N)")
        x = synth.token_bank(x, w, args.resident_frac, host_backing=args.host_backing, poison=0.0)
        bank = {"k_backing": x["k_backing"], "touched": torch.zeros_like(x["page_table"], dtype=torch.uint8)}
        bank_attn = {"k_backing": x["k_backing"], "v_backing": x["v_backing"],
                     "touched": torch.zeros_like(x["page_table"], dtype=torch.uint8)}
        w = synth.scaled(w, name=f"{w.name}_bank{args.resident_frac:g}{'_host' if args.host_backing else ''}")
    idx = torch.empty((w.batch, w.n_q_heads, w.n_query_blocks, w.kb), dtype=torch.int32, device="cuda")
    out = torch.empty_like(x["Q"])

    # scratch of the top-r pre-pass (a copy of Q), allocated once outside the timed region
    ws = torch.empty(x["Q"].numel() * x["Q"].element_size(), dtype=torch.uint8, device="cuda") if args.top_r else None
    refresh = max(1, args.refresh_period) if w.q_len < w.kv_len else 1
    n_e = max(1, args.n_e)
    k_attn = w.k
    if n_e > 1:
        # ensemble of masks: n_e samples and a vote per step; the attention then runs over the merged list
        width = w.kb if args.tau else n_e * w.kb
        k_attn = width * w.bk
        idx = torch.empty((w.batch, w.n_q_heads, w.n_query_blocks, width), dtype=torch.int32, device="cuda")
        ws_e = torch.empty(n_e * w.batch * w.n_q_heads * w.n_query_blocks * w.kb * 4 + 256, dtype=torch.uint8, device="cuda")

    def run_mask():
        if n_e > 1:
            hipattn.hip_mask_ensemble(x["Q"], x["K"], w.k, w.bq, w.bk, n_e, args.theta_vote, args.tau, 1234, args.r_e,
                                      kv_lens=x["kv_lens"], page_table=x["page_table"], max_kv_len=max_len, flags=flags,
                                      b_sq=args.b_sq, b_sk=args.b_sk, rep_pos=args.rep_pos, workspace=ws_e, indices=idx)
            return
        hipattn.hip_mask_estimate(x["Q"], x["K"], w.k, w.bq, w.bk, kv_lens=x["kv_lens"], page_table=x["page_table"],
                                  max_kv_len=max_len, flags=flags, indices=idx, b_sq=args.b_sq, b_sk=args.b_sk,
                                  rep_pos=args.rep_pos, top_r=args.top_r, workspace=ws, **bank)

    def run_attn():
        hipattn.hip_sparse_attn(x["Q"], x["K"], x["V"], idx, k_attn, w.bq, w.bk, kv_lens=x["kv_lens"],
                                page_table=x["page_table"], max_kv_len=max_len, flags=flags, out=out,
                                n_sink=args.n_sink, n_window=args.n_window, **(bank_attn if bank else {}))

    for i in range(warmup):
        if i % refresh == 0:
            run_mask()
        run_attn()
    torch.cuda.synchronize()
    # events are recorded on torch's current stream, the stream the kernels are launched on
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        ev[i][0].record()
        if i % refresh == 0:
            run_mask()
        ev[i][1].record()
        run_attn()
        ev[i][2].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_step = wall * 1e3 / steps
    t_mask = sorted(e[0].elapsed_time(e[1]) for i, e in enumerate(ev) if i % refresh == 0)   # per launch
    t_attn = sorted(e[1].elapsed_time(e[2]) for e in ev)
    ms_mask, ms_attn = sum(t_mask) / len(t_mask), sum(t_attn) / len(t_attn)

    size = 2 if w.dtype == "bf16" else 4
    mask_bytes = n_e * mask_algorithmic_bytes(w, kv_lens, args.rep_pos)
    mask_flops = n_e * mask_score_flops(w, kv_lens, args.rep_pos, max(args.b_sq, 1), max(args.b_sk, 1))
    # (ensemble: the merged list is at most k_attn keys long; its real length depends on the data, so the
    # attention's algorithmic figures are upper bounds there)
    attn_flops, attn_bytes = attn_algorithmic(synth.scaled(w, k=k_attn), kv_lens)
    mask_gbs = mask_bytes / (ms_mask * 1e-3) / 1e9
    mask_tflops = mask_flops / (ms_mask * 1e-3) / 1e12
    attn_tflops = attn_flops / (ms_attn * 1e-3) / 1e12
    attn_gbs = attn_bytes / (ms_attn * 1e-3) / 1e9
    prefill = w.q_len > 1
    # what the gather probe sustains on a buffer the size of the rows each kernel draws from (K; K and V)
    kv_bytes = sum(int(n) for n in (kv_lens if kv_lens is not None else [w.kv_len] * w.batch)) * w.n_kv_heads * w.head_dim * size
    probe_k = probe_kv = None
    if args.gather_probe and w.head_dim * size == 256:
        probe_k = gather_ceiling(kv_bytes, w.bk)
        probe_kv = gather_ceiling(2 * kv_bytes, w.bk)

    def cand(achieved, peak, unit, **extra):
        return {"achieved": achieved, "peak": peak, "unit": unit, "frac": achieved / peak, **extra}

    def kernel_report(kernel, ms):
        """Every candidate roof of one kernel, and the one that binds."""
        traffic, tsrc = read_traffic(f"{kernel}_{tag}")
        c = {}
        if kernel == "mask_estimate":
            # bytes side: every scored key row passes L2 -> compute unit once (algorithmic bytes); whether it also
            # passes HBM -> L2 depends on the working set, so the HBM fraction by algorithmic bytes is a candidate
            # that only binds when it stays a fraction (decode over GBs of keys), and the HBM-side counter bytes of
            # an earlier profile run, when current, give the memory-side rate
            c["hbm_algorithmic"] = cand(mask_gbs, HBM_PEAK_GBS, "GB/s", bound="hbm")
            c["l2_fill_algorithmic"] = cand(mask_gbs, L2_PEAK_GBS, "GB/s", bound="l2")
            if prefill and w.dtype == "bf16":
                c["mfma_score_flops"] = cand(mask_tflops, MFMA_BF16_PEAK_TFLOPS, "TFLOP/s", bound="mfma")
            probe = probe_k
        else:
            if prefill and w.dtype == "bf16":
                c["mfma_algorithmic"] = cand(attn_tflops, MFMA_BF16_PEAK_TFLOPS, "TFLOP/s", bound="mfma")
            c["hbm_algorithmic"] = cand(attn_gbs, HBM_PEAK_GBS, "GB/s", bound="hbm")
            c["l2_fill_algorithmic"] = cand(attn_gbs, L2_PEAK_GBS, "GB/s", bound="l2")
            probe = probe_kv
        if traffic:
            c["hbm_counter"] = cand(traffic / (ms * 1e-3) / 1e9, HBM_PEAK_GBS, "GB/s", bound="hbm", source=tsrc)
        # the sparse attention of a prefill is priced as the contraction it is (bf16 MFMA peak); the other kernels
        # against whichever candidate binds
        name = "mfma_algorithmic" if "mfma_algorithmic" in c else pick_roof(c)
        roof = {"kernel": kernel, "bound": c[name]["bound"], "achieved": c[name]["achieved"], "peak": c[name]["peak"],
                "unit": c[name]["unit"], "frac": c[name]["frac"], "basis": name,
                "traffic": traffic, "traffic_source": tsrc, "ceilings": c}
        if kernel == "sparse_attn" and prefill and w.dtype == "bf16":
            # attainable matrix rate of the gather-fed contraction: bq flop per gathered byte, and every gathered byte
            # passes L2 -> compute unit, whose published fill rate therefore bounds it whatever the cache hit rates
            att = min(MFMA_BF16_PEAK_TFLOPS, w.bq * L2_PEAK_GBS / 1e3)
            roof["attainable"] = {"TFLOP/s": att, "frac_of_attainable": attn_tflops / att,
                                  "what": "min(bf16 MFMA peak, bq x L2 fill peak)"}
        if probe:
            # measured, not published, and NOT a ceiling: the same volume fetched by a kernel that does nothing else,
            # from uniformly random places (no reuse between heads or neighbouring query blocks, which the method has)
            gbs = mask_gbs if kernel == "mask_estimate" else attn_gbs
            roof["uniform_gather_reference"] = {"GB/s": probe, "ratio": gbs / probe,
                                                "what": "reuse-free gather of 512-byte runs over a buffer of this kernel's "
                                                        "working set (8 slices, one per XCD), measured in this run"}
        return roof

    roofs = {"mask_estimate": kernel_report("mask_estimate", ms_mask), "sparse_attn": kernel_report("sparse_attn", ms_attn)}
    roof = roofs["mask_estimate"] if ms_mask >= ms_attn else roofs["sparse_attn"]

    if w.q_len < w.kv_len:  # decode: one (or, for speculative decoding, a few) new rows per sequence
        metric, unit, value, hib = f"HiP decode us/step @{w.kv_len // 1024}k ctx", "us/step", ms_step * 1e3, False
    else:
        metric, unit, value, hib = (f"HiP prefill tokens/s @T={w.kv_len // 1024}k", "tokens/s",
                                    w.batch * w.q_len / (ms_step * 1e-3), True)
    res = {
        "metric": metric, "value": value, "unit": unit, "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_step, "higher_is_better": hib, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads,
                   "head_dim": w.head_dim, "q_len": w.q_len, "kv_len": w.kv_len, "k": w.k, "bq": w.bq, "bk": w.bk,
                   "kernels": "generic" if args.generic else "tuned", "b_sq": args.b_sq, "b_sk": args.b_sk, "rep_pos": args.rep_pos, "top_r": args.top_r,
                   "n_sink": args.n_sink, "n_window": args.n_window, "refresh_period": refresh,
                   "ensemble": {"n_e": n_e, "theta_vote": args.theta_vote, "tau": args.tau, "r_e": args.r_e} if n_e > 1 else None},
        "kernel_ms": {"mask_estimate": ms_mask, "sparse_attn": ms_attn},
        "kernel_ms_median": {"mask_estimate": t_mask[len(t_mask) // 2], "sparse_attn": t_attn[len(t_attn) // 2]},
        "kernel_ms_min": {"mask_estimate": t_mask[0], "sparse_attn": t_attn[0]},
        "mask_estimate": {"algorithmic_GB": mask_bytes / 1e9, "GB/s": mask_gbs, "score_TFLOP": mask_flops / 1e12,
                          "score_TFLOP/s": mask_tflops, "roofline": roofs["mask_estimate"]},
        "sparse_attn": {"algorithmic_TFLOP": attn_flops / 1e12, "TFLOP/s": attn_tflops,
                        "gathered_GB": attn_bytes / 1e9, "GB/s": attn_gbs, "roofline": roofs["sparse_attn"]},
        "roofline": {k: v for k, v in roof.items()},
    }
    if bank:
        # what the maps of pages read say: share of the sequences' pages each call touched, and how many of those missed
        table = x["page_table"]
        stats = {}
        for name, t in (("mask_estimate", bank["touched"]), ("sparse_attn", bank_attn["touched"])):
            read = t.bool()
            stats[name] = {"pages_read": int(read.sum()), "misses": int((read & (table < 0)).sum())}
        res["token_bank"] = {"resident_frac": args.resident_frac, "backing": "host" if args.host_backing else "hbm",
                             "pages_used": sum(-(-int(n) // w.page_size) for n in (kv_lens if kv_lens is not None else [w.kv_len] * w.batch)),
                             **stats}
    if args.dense_yardstick and w.q_len == w.kv_len and w.kv_len <= 131072 and not w.page_size:
        res["dense_yardstick"] = dense_yardstick(w, x)
    if with_cpu and args.cpu_budget > 0:
        res["cpu_baseline"] = cpu_baseline(w, x_plain, args.cpu_budget, n_sink=args.n_sink, n_window=args.n_window,
                                           b_sq=args.b_sq, b_sk=args.b_sk, rep_pos=args.rep_pos, top_r=args.top_r)
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c2", choices=["c1", "c2", "c3", "c4", "c5", "pd", "ps"])
    ap.add_argument("--cpu-budget", type=float, default=15.0, help="seconds of oracle time; 0 disables")
    ap.add_argument("--generic", action="store_true", help="force the shape-generic kernels")
    ap.add_argument("--no-shared-round", action="store_true",
                    help="prefill mask estimation: every head gathers the first round's key tiles itself (A/B measurement)")
    ap.add_argument("--b-sq", type=int, default=1, help="query-row sampling stride of the block score (default: all rows)")
    ap.add_argument("--b-sk", type=int, default=1, help="key sampling stride of the block score (default: all keys)")
    ap.add_argument("--rep-pos", type=int, default=0, choices=[0, 1, 2],
                    help="representative block of a branch: 0 centre (default), 1 first, 2 last")
    ap.add_argument("--top-r", type=int, default=0,
                    help="score over each query row's top-r channels only (default 0: all channels)")
    ap.add_argument("--n-sink", type=int, default=0, help="sink keys added in the sparse attention (default 0)")
    ap.add_argument("--n-window", type=int, default=0, help="sliding-window keys added in the sparse attention (default 0)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one 1 GiB device copy (counter calibration for rocprofv3 --pmc runs)")
    ap.add_argument("--seq-len", type=int, default=0,
                    help="override the workload's context length (prefill: also its query length); scaling studies")
    ap.add_argument("--refresh-period", type=int, default=1,
                    help="decode only: estimate the mask every R-th step and reuse it in between (Alg. 2's mask "
                         "refresh period); combine with --n-window >= R so that the newest keys stay attended")
    ap.add_argument("--q-len", type=int, default=0,
                    help="query rows per sequence, placed at the end of the context (chunked prefill, speculative decoding)")
    ap.add_argument("--k", type=int, default=0, help="override the workload's k (a multiple of its bk)")
    ap.add_argument("--page-size", type=int, default=-1,
                    help="override the KV layout: tokens per page of a paged pool (a multiple of bk), 0 = contiguous")
    ap.add_argument("--resident-frac", type=float, default=-1.0,
                    help="token bank (paged workloads): house this fraction of the pages in a bank of resident pages and "
                         "read the others through negative page-table entries from a backing pool; both calls also "
                         "write their map of pages read (default: off)")
    ap.add_argument("--host-backing", action="store_true", help="with --resident-frac: the backing pool lives in pinned host memory")
    ap.add_argument("--bk", type=int, default=0, help="override the workload's key block size")
    ap.add_argument("--bq", type=int, default=0, help="override the workload's query block size")
    ap.add_argument("--peaks", action="store_true",
                    help="also measure what this GPU sustains on a 1 GiB device copy and on back-to-back bf16 MFMAs")
    ap.add_argument("--dense-yardstick", action="store_true",
                    help="also time torch's dense causal attention on the same tensors (prefill workloads up to "
                         "128k tokens; external yardstick, not part of the path)")
    ap.add_argument("--n-e", type=int, default=1,
                    help="ensemble of masks: samples per step (default 1: the plain mask); the vote is part of the mask time")
    ap.add_argument("--theta-vote", type=int, default=1, help="ensemble: votes a key block needs (1 = union)")
    ap.add_argument("--tau", type=int, default=0, choices=[0, 1], help="ensemble: 1 truncates the merged list to k by votes")
    ap.add_argument("--r-e", type=float, default=5.0, help="ensemble: size of the score perturbation")
    ap.add_argument("--no-gather-probe", dest="gather_probe", action="store_false",
                    help="skip the gather probe (the measured ceiling quoted next to the published ones)")
    ap.add_argument("--target-points", type=int, default=-1, choices=[-1, 0, 1],
                    help="also time the two points the targets are stated at (C2's shape at T = 131072, C3 decode at "
                         "128k context) and add them as `target_points`; default: on for the plain default run only")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding or collectives are part of it); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    torch.cuda.set_device(0)
    plain = (args.k == 0 and args.bk == 0 and args.bq == 0 and args.q_len == 0 and args.page_size < 0
             and args.resident_frac < 0 and not args.generic and args.b_sq <= 1 and args.b_sk <= 1 and args.rep_pos == 0
             and args.top_r == 0 and args.n_sink == 0 and args.n_window == 0 and args.refresh_period <= 1
             and args.n_e <= 1 and not args.no_shared_round)

    def tag_of(workload, seq_len):
        # counter summaries under profiles/ exist for the named workloads as they stand and for C2's shape at 128k
        if not plain:
            return "none"
        if seq_len == 0:
            return workload
        return "c2_128k" if (workload == "c2" and seq_len == 131072) else "none"

    if args.calib_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    w = build_workload(args)
    res = measure(args, w, tag_of(args.workload, args.seq_len), args.steps, args.warmup, with_cpu=True)
    res["kernel_source_sha"] = kernel_source_sha()
    want_points = args.target_points == 1 or (args.target_points == -1 and plain and args.workload == "c2" and args.seq_len == 0)
    if want_points:
        points = {}
        for name, seq_len in (("c2", 131072), ("c3", 0)):
            torch.cuda.empty_cache()
            r = measure(args, build_workload(args, name, seq_len), tag_of(name, seq_len), min(args.steps, 10),
                        min(args.warmup, 3), with_cpu=False)
            points["c2_T131072" if name == "c2" else "c3"] = {
                k: r[k] for k in ("metric", "value", "unit", "steps", "warmup", "ms_per_step", "config", "kernel_ms",
                                  "kernel_ms_median", "kernel_ms_min", "mask_estimate", "sparse_attn")}
        res["target_points"] = points
    if args.peaks:
        res["measured_peaks"] = measured_peaks()
    print(json.dumps(res))


if __name__ == "__main__":
    main()
