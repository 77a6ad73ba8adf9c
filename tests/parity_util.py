"""Shared plumbing of the GPU parity tests: upload, run the HIP stage through the C ABI,
run the fp64 oracle on the same stored inputs, compare by the parity rules.

Parity rules (tolerances derived in the design notes):
  * index work (top-k given a score, positions, K/V rows, copied hidden rows): bit-exact;
  * kept set vs the end-to-end oracle: identical, except indices whose oracle score lies
    within 1e-6 (relative) of the k-th score;
  * routing: identical, except where the oracle's similarity gap between its choice and the
    GPU's is below 1e-5;
  * merged rows: |d| <= tol * max(|ref|, rms(ref row)) and ||d||2 <= tol ||ref||2 with
    tol = 1e-4 (f32) / 2e-2 (bf16);
  * when a tolerated tie changes a discrete result, what follows is judged stage-wise: the
    oracle step is re-run on the GPU's discrete outputs.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

from oracle import asap_oracle as O
from paper_2603_14549_amd import binding, harness, synth

TOL = {"f32": 1e-4, "bf16": 2e-2}
TIE_REL = 1e-6
ROUTE_GAP = 1e-5


to_device = harness.to_device


def from_device(t: torch.Tensor) -> np.ndarray:
    """-> float64 (floating tensors, exact upcast) or the integer array."""
    t = t.detach().cpu()
    if t.dtype == torch.bfloat16:
        return t.float().numpy().astype(np.float64)
    if t.dtype == torch.float32:
        return t.numpy().astype(np.float64)
    return t.numpy()


def raw_bits(t: torch.Tensor) -> np.ndarray:
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype == torch.float32:
        return t.view(torch.int32).numpy().view(np.uint32)
    return t.numpy()


GpuStage = harness.DeviceStage


def oracle_image(inp: dict, b: int, lambda_max=1.0, eps=1e-6, mask_on=True, mu=1.0, threshold=None,
                 lse_extra: Optional[np.ndarray] = None, linear_mass: Optional[bool] = None,
                 score_rows: str = "all") -> dict:
    cfg = inp["cfg"]
    Q = synth.to_f64(inp["q"][b], cfg.qk_dtype)
    K = synth.to_f64(inp["k"][b], cfg.qk_dtype)
    X = synth.to_f64(inp["hidden"][b], cfg.h_dtype)
    if linear_mass is None:
        linear_mass = cfg.V > 600          # the explicit V x V form is kept for the smaller cases
    return O.stage(Q, K, X, int(inp["text_len"][b]), cfg.P, cfg.V, cfg.Tmax, cfg.k, lambda_max=lambda_max,
                   eps=eps, mask_on=mask_on, mu=mu, threshold=threshold,
                   lse_extra=None if lse_extra is None else lse_extra[b].astype(np.float64),
                   linear_mass=linear_mass, score_rows=score_rows)


def check_rows(got: np.ndarray, ref: np.ndarray, tol: float, what: str):
    """Row-wise relative L2 and element-wise bound against max(|ref|, rms(row))."""
    d = got - ref
    rms = np.sqrt((ref * ref).mean(axis=1, keepdims=True))
    bound = tol * np.maximum(np.abs(ref), rms)
    bad = np.abs(d) > bound + 1e-30
    assert not bad.any(), f"{what}: {bad.sum()} elements off, worst ratio {np.max(np.abs(d) / (bound + 1e-30)):.3g}"
    l2 = np.sqrt((d * d).sum(axis=1)) / np.maximum(np.sqrt((ref * ref).sum(axis=1)), 1e-30)
    assert l2.max() <= tol, f"{what}: row relative L2 {l2.max():.3g} > {tol}"


def compare_image(inp: dict, buf, b: int, ref: dict, mu=1.0, threshold=-math.inf, report: Optional[dict] = None):
    """All parity checks of image b.  `ref` = oracle_image(...) with the same parameters."""
    cfg = inp["cfg"]
    P, V, k, Tmax, D = cfg.P, cfg.V, cfg.k, cfg.Tmax, cfg.D
    M = V - k
    tl = int(inp["text_len"][b])
    tol = TOL[cfg.h_dtype]
    X = synth.to_f64(inp["hidden"][b], cfg.h_dtype)
    Xv = X[P:P + V]

    # ---- Eq. 2-3: mass and salience (fp64 sums on the GPU, one rounding to f32)
    s_raw = from_device(buf.s_raw[b])
    s_hat = from_device(buf.s_hat[b])
    smax = np.abs(ref["s_raw"]).max()
    # one f32 rounding of s (6e-8 |s|) plus the fp32 sums of a head's products inside the matrix
    # instruction: their error scales with the heads' partial sums, which cancel in s when heads
    # disagree in sign (images with two or three visual tokens show it)
    Qf = synth.to_f64(inp["q"][b], cfg.qk_dtype)[:, P:P + V]
    Kf = synth.to_f64(inp["k"][b], cfg.qk_dtype)[:, P:P + V]
    qbar = np.zeros((cfg.Hkv, cfg.d))
    for h in range(cfg.H):
        qbar[(h * cfg.Hkv) // cfg.H] += Qf[h].sum(axis=0)
    head_scale = np.abs(np.einsum("gd,gjd->gj", qbar, Kf)).sum(axis=0).max() / (cfg.H * math.sqrt(cfg.d))
    s_tol = 2e-7 * max(smax, 0.6 * head_scale) + 1e-30
    assert np.abs(s_raw - ref["s_raw"]).max() <= s_tol, "s_raw"
    assert np.abs(s_hat - ref["s_hat"]).max() <= 2e-7, "s_hat"

    # ---- Eq. 5 -> selection score
    score = from_device(buf.score[b])
    r = ref["score"]
    rel = np.abs(score - r) / np.maximum(r, 1e-9 * r.max())
    if report is not None:
        report.setdefault("score_rel_err", []).append(float(rel.max()))
    # 2e-5 for the softmax terms, plus what the tolerance of s (2e-7 max|s| absolute, checked above, on
    # s_j and on the minimum alike) becomes after Eq. 3-4: the score is proportional to lambda'_j, i.e.
    # to s_j - min s, so keys whose mass is close to the image's minimum feel it most
    s64 = ref["s_raw"]
    bound = 2e-5 + 2 * 2e-7 * smax / np.maximum(s64 - s64.min(), 1e-300)
    assert (rel <= bound).all(), f"score: relative error {rel.max():.3g}, worst excess {(rel / bound).max():.3g} x bound"
    assert abs(score.sum() - r.sum()) <= 1e-5

    # ---- top-k: exact given the GPU's own score (integer work) ...
    kept = buf.kept_idx[b].cpu().numpy().astype(np.int64)
    pruned = buf.pruned_idx[b].cpu().numpy().astype(np.int64)[:M]
    k_ref, p_ref = O.select_topk(buf.score[b].cpu().numpy().astype(np.float64), k)
    assert (kept == k_ref).all() and (pruned == p_ref).all(), "top-k of the GPU score is not exact"
    # ... and against the end-to-end oracle: identical up to ties below 1e-6 relative
    same_kept = (kept == ref["kept"]).all()
    if not same_kept:
        r_sorted = np.sort(r)[::-1]
        r_k = r_sorted[k - 1]
        diff = np.setxor1d(kept, ref["kept"])
        gaps = np.abs(r[diff] - r_k) / r_k
        assert gaps.max() < TIE_REL, f"kept set differs beyond ties: gaps {gaps}"
    if report is not None:
        report.setdefault("kept_equal", []).append(bool(same_kept))

    # ---- routing, stage-wise on the GPU's index sets
    if M > 0:
        assign = buf.assign[b].cpu().numpy().astype(np.int64)[:M]
        best = from_device(buf.best_sim[b])[:M]
        C = O.cosine_matrix(Xv[pruned], Xv[kept])
        a_ref = np.argmax(C, axis=1)
        b_ref = C[np.arange(M), a_ref]
        assert np.abs(best - b_ref).max() <= 2e-5, f"best_sim off by {np.abs(best - b_ref).max():.3g}"
        routed_ref = b_ref > threshold
        routed = assign >= 0
        flip = routed != routed_ref
        if flip.any():      # only legitimate right at the threshold
            assert np.abs(b_ref[flip] - threshold).max() < ROUTE_GAP
        both = routed & routed_ref
        differ = both & (assign != a_ref)
        if differ.any():
            gap = b_ref[differ] - C[np.nonzero(differ)[0], assign[differ]]
            assert gap.max() < ROUTE_GAP, f"assign differs beyond near-ties: gap {gap.max():.3g}"
        if report is not None:
            report.setdefault("assign_mismatch", []).append(int(differ.sum()))
    else:
        assign = np.zeros(0, dtype=np.int64)

    # ---- Eq. 6 on the GPU's discrete outputs, salience from the oracle
    sources = O.sources_from_assign(assign, pruned, k)
    y_ref, w_ref = O.weighted_merge(Xv, ref["s_hat"], kept, sources, mu)
    Y_ref, pos_ref, nl_ref = O.assemble_sequence(X, y_ref, kept, P, V, Tmax, tl)
    Y = from_device(buf.out_hidden[b])
    pos = buf.pos_out[b].cpu().numpy().astype(np.int64)
    assert int(buf.new_len[b]) == nl_ref
    assert (pos == pos_ref).all(), "pos_out"
    assert (buf.final_idx[b].cpu().numpy() == kept).all(), "final_idx"
    wsum = from_device(buf.wsum[b])
    assert np.abs(wsum - w_ref).max() <= 1e-5 * max(1.0, np.abs(w_ref).max()), "wsum"
    check_rows(Y[P:P + k], Y_ref[P:P + k], tol, "merged rows")
    # prefix, text, and slots that absorbed nothing are bit-exact copies
    got_bits = raw_bits(buf.out_hidden[b])
    src_bits = inp["hidden"][b]
    if src_bits.dtype == np.float32:
        src_bits = src_bits.view(np.uint32)
    assert (got_bits[:P] == src_bits[:P]).all(), "prefix rows"
    assert (got_bits[P + k:nl_ref] == src_bits[P + V:P + V + tl]).all(), "text rows"
    absorbed = np.array([mu * ref["s_hat"][s].sum() if s.size else 0.0 for s in sources])
    lone = np.nonzero(absorbed == 0.0)[0]
    assert (got_bits[P + lone] == src_bits[P + kept[lone]]).all(), "slots without sources"

    # ---- K/V rows, bit-exact
    for l in range(len(buf.k_dst)):
        for dst, src in ((buf.k_dst[l], inp["k_cache"][l]), (buf.v_dst[l], inp["v_cache"][l])):
            got = raw_bits(dst[b])
            s = src[b]
            if s.dtype == np.float32:
                s = s.view(np.uint32)
            want = s[:, pos_ref[:nl_ref], :]
            assert (got[:, :nl_ref] == want).all(), f"K/V rows of layer {l}"

    # ---- end to end, when no tie intervened
    if same_kept and M > 0:
        check_rows(Y[P:P + k], ref["Y"][P:P + k], tol * 1.0, "merged rows end-to-end") if (
            (assign == ref["assign"]).all()) else None
    return same_kept


def compare_image_paper(inp: dict, buf, b: int, threshold: float, mu: float = 1.0) -> dict:
    """Parity of image b with ASAP_ROUTE_PAPER.  The routing is judged stage-wise: the oracle's
    route_paper runs on the GPU's own kept / pruned sets and on the GPU's f32 s_hat, s_raw (the
    predicates s_hat_i > s_hat_j and the refill order are decisions taken in that precision); what
    follows (Eq. 6, output sequence, K/V rows) is then compared as for the other route."""
    cfg = inp["cfg"]
    P, V, k, Tmax = cfg.P, cfg.V, cfg.k, cfg.Tmax
    tl = int(inp["text_len"][b])
    tol = TOL[cfg.h_dtype]
    X = synth.to_f64(inp["hidden"][b], cfg.h_dtype)
    Xv = X[P:P + V]
    kept = buf.kept_idx[b].cpu().numpy().astype(np.int64)
    pruned = buf.pruned_idx[b].cpu().numpy().astype(np.int64)[:V - k]
    s_hat = from_device(buf.s_hat[b])
    s_raw = from_device(buf.s_raw[b])
    final_ref, sources_ref = O.route_paper(Xv, s_raw, s_hat, kept, pruned, threshold)
    final = buf.final_idx[b].cpu().numpy().astype(np.int64)
    assign = buf.assign.flatten()[b * k:(b + 1) * k].cpu().numpy().astype(np.int64)
    best = from_device(buf.best_sim.flatten()[b * k:(b + 1) * k])

    # immediate destinations: best stronger kept token above the threshold
    C = O.cosine_matrix(Xv[kept], Xv[kept])
    sh_k = s_hat[kept]
    stronger = (sh_k[:, None] > sh_k[None, :]) | ((sh_k[:, None] == sh_k[None, :]) &
                                                   (np.arange(k)[:, None] < np.arange(k)[None, :]))   # [dest, src]
    Cm = np.where(stronger, C, -np.inf)
    b_ref = Cm.max(axis=0)
    has = np.isfinite(b_ref)
    assert (np.isfinite(best) == has).all(), "which kept tokens have a stronger neighbour at all"
    assert np.abs(best[has] - b_ref[has]).max(initial=0.0) <= 2e-5, "best_sim (paper route)"
    near = has & (np.abs(b_ref - threshold) < ROUTE_GAP)        # decisions right at the threshold may flip
    assert not near.any(), "test input has a similarity within 1e-5 of the threshold; pick another threshold"

    assert final.shape == final_ref.shape and (final == final_ref).all(), "final_idx"
    assert (np.diff(final) > 0).all()
    sources = [kept[assign == c] for c in range(k)]
    for c in range(k):
        assert (sources[c] == sources_ref[c]).all(), f"sources of final slot {c}"
    surv = assign < 0
    assert set(kept[surv]).issubset(set(final.tolist())), "a surviving kept token is missing from final_idx"
    n_sources = int((~surv).sum())
    refill = np.setdiff1d(final, kept)
    assert refill.size == n_sources, "one refill per vacated slot"

    y_ref, w_ref = O.weighted_merge(Xv, s_hat, final, sources, mu)
    Y_ref, pos_ref, nl_ref = O.assemble_sequence(X, y_ref, final, P, V, Tmax, tl)
    Y = from_device(buf.out_hidden[b])
    pos = buf.pos_out[b].cpu().numpy().astype(np.int64)
    assert int(buf.new_len[b]) == nl_ref
    assert (pos == pos_ref).all(), "pos_out"
    wsum = from_device(buf.wsum[b])
    assert np.abs(wsum - w_ref).max() <= 1e-5 * max(1.0, np.abs(w_ref).max()), "wsum"
    check_rows(Y[P:P + k], Y_ref[P:P + k], tol, "merged rows (paper route)")
    got_bits = raw_bits(buf.out_hidden[b])
    src_bits = inp["hidden"][b]
    if src_bits.dtype == np.float32:
        src_bits = src_bits.view(np.uint32)
    assert (got_bits[:P] == src_bits[:P]).all(), "prefix rows"
    assert (got_bits[P + k:nl_ref] == src_bits[P + V:P + V + tl]).all(), "text rows"
    absorbed = np.array([mu * s_hat[s].sum() if s.size else 0.0 for s in sources])
    lone = np.nonzero(absorbed == 0.0)[0]
    assert (got_bits[P + lone] == src_bits[P + final[lone]]).all(), "slots without sources"
    for l in range(len(buf.k_dst)):
        for dst, src in ((buf.k_dst[l], inp["k_cache"][l]), (buf.v_dst[l], inp["v_cache"][l])):
            got = raw_bits(dst[b])
            s = src[b]
            if s.dtype == np.float32:
                s = s.view(np.uint32)
            assert (got[:, :nl_ref] == s[:, pos_ref[:nl_ref], :]).all(), f"K/V rows of layer {l}"
    return {"n_sources": n_sources, "n_refill": int(refill.size)}


def run_and_compare(cfg, images: Optional[Sequence[int]] = None, lse=False, ctx=None, report=None,
                    last_token=False, **param_overrides):
    """Generate, run on the GPU, compare the chosen images (all by default)."""
    inp = synth.make_inputs(cfg)
    lse_extra = None
    if lse:
        rng = np.random.default_rng(cfg.seed + 77)
        lse_extra = rng.normal(2.0, 2.0, size=(cfg.B, cfg.H, cfg.Tmax)).astype(np.float32)
    stage = GpuStage(inp, ctx=ctx, lse_extra=lse_extra, last_token=last_token, **param_overrides)
    buf = stage.run()
    mask_on = param_overrides.get("mask_mode", binding.ASAP_MASK_KEYBIAS) == binding.ASAP_MASK_KEYBIAS
    mu = param_overrides.get("merge_weight", 1.0)
    thr = param_overrides.get("sim_threshold", -math.inf)
    lam = param_overrides.get("lambda_max", 1.0)
    eps = param_overrides.get("eps", 1e-6)
    for b in (range(cfg.B) if images is None else images):
        ref = oracle_image(inp, b, lambda_max=lam, eps=float(np.float32(eps)), mask_on=mask_on, mu=mu,
                           threshold=thr, lse_extra=lse_extra, score_rows="last" if last_token else "all")
        compare_image(inp, buf, b, ref, mu=mu, threshold=thr, report=report)
    return inp, stage
