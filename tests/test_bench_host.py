"""Host-side logic of bench.py, checked without a GPU: the one-GPU rule, the algorithmic byte counts the
roofline figures are built on, and the rule that measured traffic is only quoted from a counter summary
that lists exactly the kernels a run launched."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench                                          # noqa: E402
from paper_2603_14549_amd import synth                # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_algorithmic_bytes_of_the_benchmark_configuration():
    """Every input read once, every output written once, by hand for C6 (B = 16, P = 35, V = 2304, T = 64,
    H = Hkv = 32, d = 128, D = 4096, k = 320, two K/V layers, bf16, full text blocks)."""
    cfg = synth.CONFIGS["C6"]
    B, P, V, T, H, d, D, k, e = 16, 35, 2304, 64, 32, 128, 4096, 320, 2
    a = bench.algorithmic_bytes(cfg, float(T), 2)
    score = B * (V * d * (H + H) * e + H * T * d * e + 12 * V)
    select = B * 12 * V
    sim = B * (V * D * e + 8 * (V - k))
    merge = B * (V * D * e + (P + T) * D * e + (P + k + T) * D * e)
    kv = B * 4 * 2 * H * (P + k + T) * d * e
    assert a["stage"] == score + select + sim + merge + kv
    assert round(a["stage"] / 1e6, 1) == 1724.7
    assert a["sim_flops"] == 2.0 * B * (V - k) * k * D
    # the K/V rows that no selection changes are part of the compaction's bytes, not extra ones
    assert a["per_kernel"]["kv_fixed_rows"] == B * 4 * 2 * H * (P + T) * d * e
    assert a["per_kernel"]["k_compact"] == kv
    assert a["per_kernel"]["k_score_select_kv"] - a["per_kernel"]["k_score_select"] == a["per_kernel"]["kv_fixed_rows"]


def test_measured_traffic_is_only_quoted_for_the_kernels_the_summary_lists(tmp_path, monkeypatch):
    prof = tmp_path / "profiles"
    prof.mkdir()
    (prof / "bench_CX_hbm_traffic.txt").write_text(
        "header line\n"
        "kernel                                    FETCH KiB   WRITE KiB  fetch MB  write MB  total MB\n"
        "k_qsum<bf16_t>                               147497        1536     302.1       1.6     303.6\n"
        "k_sim<bf16_t, 5, false>                      152705         248     312.7       0.3     313.0\n"
        "sum over the kernels of one step: 616.6 MB\n")
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    table, source, note = bench.measured_traffic("CX", ["k_qsum", "k_sim"])
    assert table == {"k_qsum": 303.6e6, "k_sim": 313.0e6} and source.endswith("bench_CX_hbm_traffic.txt")
    table, _, note = bench.measured_traffic("CX", ["k_qsum", "k_sim", "k_merge"])       # a kernel the summary lacks
    assert table is None and "k_merge" in note
    table, _, note = bench.measured_traffic("CX", ["k_qsum"])                           # a kernel no longer launched
    assert table is None and "k_sim" in note
    table, _, note = bench.measured_traffic("CY", ["k_qsum"])
    assert table is None and "no counter summary" in note


def test_the_committed_counter_summaries_name_the_kernels_of_their_workloads():
    c6 = ["k_qsum", "k_mass_mfma", "k_attn_stats", "k_attn_colsum", "k_score_select_kv", "k_compact", "k_sim", "k_merge"]
    c3 = ["k_qsum", "k_mass_mfma", "k_attn_stats", "k_colsum_rows", "k_score_select", "k_compact", "k_sim_f32",
          "k_sim_reduce", "k_merge"]
    for workload, kernels in (("C6", c6), ("C3", c3)):
        table, _, note = bench.measured_traffic(workload, kernels)
        assert table is not None, (workload, note)
        assert all(v > 0 for v in table.values())
