"""Checks of the synthetic-input generator (no method arithmetic lives there)."""
import numpy as np
import torch

from paper_2603_14549_amd import synth


def test_bf16_rounding_matches_torch_rne():
    x = np.random.default_rng(0).standard_normal(100000).astype(np.float32) * 37.0
    x[:4] = [0.0, -0.0, 1.00390625, 1.01171875]        # two exact ties: round to even
    bits = synth.f32_to_bf16_bits(x)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert (bits == want).all()
    back = synth.bf16_bits_to_f32(bits)
    assert (back == torch.from_numpy(x).to(torch.bfloat16).float().numpy()).all()


def test_rope_depends_on_relative_position_only():
    # (R_m q) . (R_n k) is a function of m - n (Sec. 3.1)
    rng = np.random.default_rng(1)
    q = rng.standard_normal((1, 16)).astype(np.float64)
    k = rng.standard_normal((1, 16)).astype(np.float64)
    def score(m, n):
        return float(synth.rope_rotate(q, np.array([m]), 10000.0) @ synth.rope_rotate(k, np.array([n]), 10000.0).T)
    assert abs(score(40, 10) - score(530, 500)) < 1e-9
    assert abs(score(7, 7) - float(q @ k.T)) < 1e-12
    assert abs(score(40, 10) - score(40, 11)) > 1e-6


def test_make_inputs_shapes_determinism_and_recipe():
    cfg = synth.CONFIGS["S1"]
    a = synth.make_inputs(cfg)
    b = synth.make_inputs(cfg)
    assert a["q"].shape == (cfg.B, cfg.H, cfg.N, cfg.d) and a["q"].dtype == np.float32
    assert a["k"].shape == (cfg.B, cfg.Hkv, cfg.N, cfg.d)
    assert a["hidden"].shape == (cfg.B, cfg.N, cfg.D)
    assert len(a["k_cache"]) == cfg.L_kv and a["k_cache"][0].dtype == np.uint16
    assert a["k_cache"][0].shape == (cfg.B, cfg.Hkv, cfg.N, cfg.d)
    for key in ("q", "k", "hidden", "text_len"):
        assert (a[key] == b[key]).all()
    assert (a["k_cache"][1] == b["k_cache"][1]).all()
    assert a["text_len"].min() >= cfg.text_lo and a["text_len"].max() == cfg.Tmax
    # 8x outliers at every 64th visual token
    Xv = a["hidden"][0, cfg.P:cfg.P + cfg.V].astype(np.float64)
    norms = np.linalg.norm(Xv, axis=1)
    assert norms[0] > 5 * np.median(norms) and norms[64] > 5 * np.median(norms)
    # images draw their own centres
    assert not np.allclose(a["hidden"][0, cfg.P + 1], a["hidden"][1, cfg.P + 1])


def test_configs_match_the_benchmark_shapes():
    c = synth.CONFIGS
    assert (c["C1"].P, c["C1"].V, c["C1"].Tmax, c["C1"].k, c["C1"].N) == (35, 576, 32, 144, 643)
    assert (c["C2"].V, c["C2"].Tmax, c["C2"].k, c["C2"].qk_dtype) == (2304, 64, 320, "bf16")
    assert (c["C3"].B, c["C3"].Tmax, c["C3"].kv_dtype, c["C3"].L_kv) == (16, 128, "bf16", 2)
    assert (c["C4"].D, c["C4"].H, c["C4"].Hkv, c["C4"].V, c["C4"].k, c["C4"].B) == (3584, 28, 4, 4096, 512, 4)
    assert (c["C5a"].D, c["C5a"].H, c["C5a"].k, c["C5b"].V, c["C5b"].k, c["C5b"].B) == (5120, 40, 576, 576, 160, 8)
    assert (c["C6"].B, c["C6"].V, c["C6"].k) == (16, 2304, 320)
