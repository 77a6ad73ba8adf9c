"""asap_score_static, the scoring call that allocates nothing and takes no workspace (its scratch is
an array inside the library), against asap_score on the same inputs: two calls in a row on one
context, the second on a smaller batch, so that whatever the first call left in the shared array
is there when the second runs.  Both calls launch the same kernels there, so the three outputs must
agree bit for bit (which is inside every tolerance of the parity rules); the second call's result is
also compared with the fp64 oracle.  With f32 keys asap_score stores the text rows' logits in its
workspace when that stays moderate; where the built-in array cannot hold them the static call sweeps
the keys a second time instead, and the two agree within the parity rules, not bit for bit.
Parameters whose scratch exceeds the array are refused before anything is launched."""
import numpy as np
import pytest
import torch

import parity_util as U
from oracle import asap_oracle as O
from paper_2603_14549_amd import binding, harness, synth

pytestmark = pytest.mark.gpu


def _inputs(cfg):
    inp = synth.make_inputs(cfg, with_kv=False)
    q = harness.to_device(inp["q"], cfg.qk_dtype)
    k = harness.to_device(inp["k"], cfg.qk_dtype)
    text_len = torch.from_numpy(inp["text_len"].astype(np.int32)).cuda()
    return inp, q, k, text_len


def _score_both_ways(ctx, cfg):
    inp, q, k, text_len = _inputs(cfg)
    p = binding.params_from_config(cfg)
    P, V = cfg.P, cfg.V
    q_vis, q_txt, k_vis = q[:, :, P:P + V], q[:, :, P + V:], k[:, :, P:P + V]
    out = {}
    for which in ("static", "workspace"):
        s_raw, s_hat, score = (torch.full((cfg.B, V), float("nan"), dtype=torch.float32, device="cuda")
                               for _ in range(3))
        if which == "static":
            ctx.asap_score_static(p, q_vis, q_txt, k_vis, text_len, None, s_raw, s_hat, score)
        else:
            ws = torch.empty(binding.asap_workspace_bytes(p), dtype=torch.uint8, device="cuda")
            ctx.asap_score(p, q_vis, q_txt, k_vis, text_len, None, s_raw, s_hat, score, ws)
        torch.cuda.synchronize()
        out[which] = [t.cpu().numpy() for t in (s_raw, s_hat, score)]
    return inp, out


def _against_the_oracle(cfg, inp, outs):
    """The rules of the parity tests: salience within what the observed mass error allows through Eq. 3,
    scores 2e-5 relative away from the image's least salient keys."""
    for b in range(cfg.B):
        ref = O.stage(synth.to_f64(inp["q"][b], cfg.qk_dtype), synth.to_f64(inp["k"][b], cfg.qk_dtype),
                      synth.to_f64(inp["hidden"][b], cfg.h_dtype), int(inp["text_len"][b]), cfg.P, cfg.V,
                      cfg.Tmax, cfg.k)
        s_raw, s_hat = outs[0][b].astype(np.float64), outs[1][b].astype(np.float64)
        sh_tol = U.salience_tolerance(s_raw, s_hat, ref)
        assert np.abs(s_hat - ref["s_hat"]).max() <= sh_tol
        r = ref["score"]
        lam = np.maximum(ref["s_hat"], 1e-6)
        err = np.abs(outs[2][b] - r)
        assert (err <= 2e-5 * r + 2 * max(sh_tol, 2e-7) * (r / lam) + 1e-300).all()


def test_static_scratch_scoring_matches_the_workspace_call_twice_in_a_row():
    ctx = binding.Context(0)
    # S2: two images, 461 visual tokens (ragged last key tile), GQA, ragged text; then S0: 72 tokens, f32
    for name in ("S2", "S0"):
        cfg = synth.CONFIGS[name]
        inp, out = _score_both_ways(ctx, cfg)
        for a, b, what in zip(out["static"], out["workspace"], ("s_raw", "s_hat", "score")):
            assert np.isfinite(a).all(), (name, what)
            assert (a.view(np.uint32) == b.view(np.uint32)).all(), (name, what)
        _against_the_oracle(cfg, inp, out["static"])
    ctx.close()


def test_static_scratch_too_small_for_the_stored_logits_of_f32_keys():
    """Three images of C3's shape (f32, 576 visual tokens, up to 128 text rows): 28 MB of logits, which
    asap_score keeps in its workspace and the 16 MiB array cannot hold.  Mass and salience do not depend
    on that and agree bit for bit; the scores of both calls are held to the oracle."""
    ctx = binding.Context(0)
    cfg = synth.shrink(synth.CONFIGS["C3"], B=3)
    p = binding.params_from_config(cfg)
    assert binding.asap_workspace_bytes(p) > 16 << 20
    inp, out = _score_both_ways(ctx, cfg)
    for a, b, what in zip(out["static"][:2], out["workspace"][:2], ("s_raw", "s_hat")):
        assert (a.view(np.uint32) == b.view(np.uint32)).all(), what
    assert np.isfinite(out["static"][2]).all() and np.isfinite(out["workspace"][2]).all()
    _against_the_oracle(cfg, inp, out["static"])
    _against_the_oracle(cfg, inp, out["workspace"])
    ctx.close()


def test_static_scratch_refuses_what_does_not_fit():
    ctx = binding.Context(0)
    cfg = synth.CONFIGS["S0"]
    _, q, k, text_len = _inputs(cfg)
    # the same tensors described as a batch whose per-head column sums alone exceed the array:
    # the size check comes before any pointer is used
    p = binding.make_params(16, 64, 64, 128, 4096, 0, 16384, 128, 100, "bf16", "bf16", "bf16")
    outs = [torch.zeros(4, dtype=torch.float32, device="cuda") for _ in range(3)]
    with pytest.raises(binding.AsapError) as err:
        ctx.asap_score_static(p, q, q, k, text_len, None, *outs)
    assert err.value.status == binding.ASAP_EWORKSPACE and "asap_score_static" in str(err.value)
    torch.cuda.synchronize()
    assert all((t == 0).all() for t in outs)
    ctx.close()
