"""Host-side checks of the benchmark's accounting (no GPU): the round counts and algorithmic bytes the roofline
fractions are computed from, the choice of the roof that binds, and the staleness rule of the counter summaries."""
import os

import bench
from paper_2406_09827_amd import synth


def _sum_rounds(w):
    total = 0
    for qb in range(w.n_query_blocks):
        L = min(w.kv_len, w.kv_len - w.q_len + (qb + 1) * w.bq)
        total += bench.rounds_of(-(-L // w.bk), w.kb)
    return total


def test_round_counts_of_the_workloads():
    # per head: 16 blocks with 1 round, 32 with 2, ... for C2; 32 * sum r 2^(r-1) for C4; 8 + 32 + 96 for C1
    assert _sum_rounds(synth.C1) == 8 * 1 + 16 * 2 + 32 * 3
    assert _sum_rounds(synth.C2) == 16 * 1 + 32 * 2 + 64 * 3 + 128 * 4 + 256 * 5 + 512 * 6
    assert _sum_rounds(synth.C4) == 32 * sum(r * 2 ** (r - 1) for r in range(1, 10))
    assert bench.rounds_of(65536, 256) == 8 and bench.rounds_of(256, 256) == 0 and bench.rounds_of(257, 256) == 1


def test_algorithmic_bytes_of_c2():
    # 32 heads x (rounds x 256 KiB, the last round of a unit half as wide) + Q + indices
    w = synth.C2
    rounds = _sum_rounds(w)
    units_with_rounds = sum(1 for qb in range(w.n_query_blocks) if (qb + 1) * w.bq // w.bk > w.kb)
    want = w.n_q_heads * ((rounds * 2 * w.kb - units_with_rounds * w.kb) * w.bk * w.head_dim * 2
                          + w.q_len * w.head_dim * 2 + w.n_query_blocks * w.kb * 4)
    got = bench.mask_algorithmic_bytes(w, None)
    assert got == want and abs(got - 39.158e9) < 0.01e9
    flops, byts = bench.attn_algorithmic(w, None)
    assert abs(flops - 0.2729e12) < 0.001e12          # 4 * rows * keys * d, early blocks see fewer keys


def test_the_roof_that_binds_is_a_fraction():
    c = {"hbm_algorithmic": {"frac": 2.57}, "l2_fill_algorithmic": {"frac": 0.53}, "mfma_score_flops": {"frac": 0.27}, "x": None}
    assert bench.pick_roof(c) == "l2_fill_algorithmic"
    assert bench.pick_roof({"a": {"frac": 1.2}}) is None
    assert bench.pick_roof({"hbm_algorithmic": {"frac": 0.85}, "l2_fill_algorithmic": {"frac": 0.17}}) == "hbm_algorithmic"


def test_counter_summaries_are_dropped_when_the_kernels_changed(tmp_path, monkeypatch):
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    os.makedirs(tmp_path / "profiles")
    src = tmp_path / "paper_2406_09827_amd" / "csrc"
    os.makedirs(src)
    (src / "k.hip").write_text("// kernel v1\n")
    sha = bench.kernel_source_sha()
    (tmp_path / "profiles" / "traffic_mask_estimate_c2.txt").write_text(
        f"# comment\ncollected = 2026-01-01\nkernel_source_sha = {sha}\nhbm_bytes_per_launch = 4100000000\n")
    byts, source = bench.read_traffic("mask_estimate_c2")
    assert byts == 4.1e9 and source["measured_in_this_run"] is False and source["file"].endswith("traffic_mask_estimate_c2.txt")
    (src / "k.hip").write_text("// kernel v2\n")
    byts, source = bench.read_traffic("mask_estimate_c2")
    assert byts is None and source["stale"] is True
    assert bench.read_traffic("sparse_attn_none") == (None, None)
