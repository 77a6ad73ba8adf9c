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
                 score_rows: str = "all", route: str = "absorb") -> dict:
    cfg = inp["cfg"]
    Q = synth.to_f64(inp["q"][b], cfg.qk_dtype)
    K = synth.to_f64(inp["k"][b], cfg.qk_dtype)
    X = synth.to_f64(inp["hidden"][b], cfg.h_dtype)
    if linear_mass is None:
        linear_mass = cfg.V > 600          # the explicit V x V form is kept for the smaller cases
    return O.stage(Q, K, X, int(inp["text_len"][b]), cfg.P, cfg.V, cfg.Tmax, cfg.k, lambda_max=lambda_max,
                   eps=eps, mask_on=mask_on, mu=mu, threshold=threshold,
                   lse_extra=None if lse_extra is None else lse_extra[b].astype(np.float64),
                   linear_mass=linear_mass, score_rows=score_rows, route=route)


def check_rows(got: np.ndarray, ref: np.ndarray, tol: float, what: str):
    """Row-wise relative L2 and element-wise bound against max(|ref|, rms(row))."""
    d = got - ref
    rms = np.sqrt((ref * ref).mean(axis=1, keepdims=True))
    bound = tol * np.maximum(np.abs(ref), rms)
    bad = np.abs(d) > bound + 1e-30
    assert not bad.any(), f"{what}: {bad.sum()} elements off, worst ratio {np.max(np.abs(d) / (bound + 1e-30)):.3g}"
    l2 = np.sqrt((d * d).sum(axis=1)) / np.maximum(np.sqrt((ref * ref).sum(axis=1)), 1e-30)
    assert l2.max() <= tol, f"{what}: row relative L2 {l2.max():.3g} > {tol}"


def mass_error_bound(inp: dict, b: int, s_ref: np.ndarray) -> np.ndarray:
    """Forward error bound of the GPU's raw mass s_j (Eq. 2), per key, from the kernels' arithmetic,
    with u = 2^-24 (fp32 unit roundoff):
      * the visual queries are added eight rows at a time in fp32 and the eights in fp64: each
        component of the summed query is off by at most 7 u sum_i |q_i|;
      * the summed query enters the matrix cores as four bf16 pieces (exact to 2^-32), f32 keys as
        three (exact to 2^-27); every piece product is exact, and the 128 (or 64) products of one head
        and piece pair are added in fp32 inside the instruction, in an order the hardware does not
        document: at most (d - 1) u sum_c |qbar_c k_c| whatever the order; sums of pieces |p_0| + |p_1| + ...
        exceed |x| by less than 1 % on either side (1.02 together);
      * heads and pieces are added in fp64 (nothing to count), and the result is rounded once to f32.
    Observed errors are one to two orders of magnitude below this bound."""
    cfg = inp["cfg"]
    P, V = cfg.P, cfg.V
    u = 2.0 ** -24
    Qf = np.abs(synth.to_f64(inp["q"][b], cfg.qk_dtype)[:, P:P + V])
    Kf = synth.to_f64(inp["k"][b], cfg.qk_dtype)[:, P:P + V]
    Qs = synth.to_f64(inp["q"][b], cfg.qk_dtype)[:, P:P + V]
    G = cfg.H // cfg.Hkv
    abs_sum = Qf.sum(axis=1).reshape(cfg.Hkv, G, cfg.d).sum(axis=1)                 # sum_i |q_i| per kv head
    qbar = np.abs(Qs.sum(axis=1).reshape(cfg.Hkv, G, cfg.d).sum(axis=1))            # |sum_i q_i|
    scale = 1.0 / (cfg.H * math.sqrt(cfg.d))
    a_sum = np.einsum("gd,gjd->j", abs_sum, np.abs(Kf)) * scale
    a_bar = np.einsum("gd,gjd->j", qbar + 7 * u * abs_sum, np.abs(Kf)) * scale
    return u * np.abs(s_ref) + 7 * u * a_sum + 1.02 * (cfg.d - 1) * u * a_bar + 1e-300


def salience_tolerance(s_raw_gpu: np.ndarray, s_hat_gpu: np.ndarray, ref: dict, eps_: float = 1e-6) -> float:
    """Checks Eq. 3 on the GPU's own masses and returns the bound for |s_hat_gpu - s_hat_oracle|.
    Eq. 3, s_hat_j = (s_j - min s) / (max s - min s + eps), has slope at most 1 / (range + eps) in s_j,
    in the minimum and (times s_hat <= 1) in the range, so masses within e of the oracle's give saliences
    within 2 e / (range + eps) -- e is the mass error observed (itself held to the bound derived from
    the kernels' arithmetic), taken on the f32 values the call returns, which sit within u |s| / 2 of the
    fp64 masses the GPU's own Eq. 3 works on; the result is rounded once to f32 (u / 2).  u = 2^-24."""
    u = 2.0 ** -24
    smax = np.abs(s_raw_gpu).max()
    own_range = s_raw_gpu.max() - s_raw_gpu.min() + eps_
    own = (s_raw_gpu - s_raw_gpu.min()) / own_range
    assert np.abs(s_hat_gpu - own).max() <= 2 * u * smax / own_range + u, "s_hat is not Eq. 3 of the masses returned"
    e = np.abs(s_raw_gpu - ref["s_raw"]).max()
    rng_ = ref["s_raw"].max() - ref["s_raw"].min() + eps_
    return (2 * e + u * smax) / rng_ + u


def compare_image(inp: dict, buf, b: int, ref: dict, mu=1.0, threshold=-math.inf, report: Optional[dict] = None,
                  lam_max: float = 1.0, eps_: float = 1e-6, mask_on: bool = True):
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
    assert (np.abs(s_raw - ref["s_raw"]) <= mass_error_bound(inp, b, ref["s_raw"])).all(), "s_raw"
    sh_tol = salience_tolerance(s_raw, s_hat, ref, eps_)
    assert np.abs(s_hat - ref["s_hat"]).max() <= sh_tol, "s_hat"

    # ---- Eq. 5 -> selection score
    score = from_device(buf.score[b])
    r = ref["score"]
    err = np.abs(score - r)
    rel = err / np.maximum(r, 1e-9 * r.max())
    if report is not None:
        report.setdefault("score_rel_err", []).append(float(rel.max()))
    # Two sources of error.  The softmax terms: 2e-5 of the score itself.  The discount lambda'_j of
    # Eq. 4: the score is lambda'_j times the weight w_j = r_j / lambda'_j the key gets undiscounted, and
    # lambda'_j = lambda_max s_hat_j carries the error of s_hat_j (sh_tol, checked above); the rows'
    # denominators carry a weighted mean of the same relative errors over the other keys, hence the
    # factor two.  An absolute bound: small for every key, but for keys whose salience is itself near
    # 1e-6 a large share of their (tiny) score.
    lam = np.maximum(lam_max * ref["s_hat"], eps_) if mask_on else np.ones_like(r)
    bound = 2e-5 * r + 2 * max(sh_tol, 2e-7) * lam_max * (r / lam)
    assert (err <= bound + 1e-300).all(), f"score: worst excess {(err / (bound + 1e-300)).max():.3g} x bound"
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


def compare_image_paper_end_to_end(inp: dict, buf, b: int, threshold: float, mu: float = 1.0) -> dict:
    """ASAP_ROUTE_PAPER against the oracle's whole stage in fp64 (nothing of the GPU's fed back in):
    the final list and every source set must be the oracle's.  A difference is accepted only if the
    oracle's own numbers show a decision too close to call in the GPU's precision:
      * the kept sets differ by score ties below 1e-6 relative (the rule of the other route);
      * two kept tokens closer than 1e-5 in cosine to the threshold or to each other's claim on a
        source (the routing rule of the other route);
      * two kept tokens with cosine above the threshold (within 1e-5) whose saliences differ by less
        than one f32 unit (the GPU compares saliences as f32 numbers);
      * the refill boundary: raw masses of the last token taken and the first left closer than the
        error bound of s_raw.
    Returns what was found, so that callers can insist on exact agreement where the inputs have no
    such close calls."""
    cfg = inp["cfg"]
    P, V, k = cfg.P, cfg.V, cfg.k
    ref = oracle_image(inp, b, mu=mu, threshold=threshold, route="paper")
    kept = buf.kept_idx[b].cpu().numpy().astype(np.int64)
    final = buf.final_idx[b].cpu().numpy().astype(np.int64)
    assign = buf.assign.flatten()[b * k:(b + 1) * k].cpu().numpy().astype(np.int64)
    sources = [kept[assign == c] for c in range(k)]
    same_kept = bool((kept == ref["kept"]).all())
    same = same_kept and bool((final == ref["final_idx"]).all()) and \
        all((sources[c] == ref["sources"][c]).all() for c in range(k))
    out = {"same_kept": same_kept, "same": same, "close_calls": []}
    if same:
        # same discrete plan: the merged sequence must agree end to end as well
        tol = TOL[cfg.h_dtype]
        Y = from_device(buf.out_hidden[b])
        check_rows(Y[P:P + k], ref["Y"][P:P + k], tol, "merged rows end to end (paper route)")
        assert (buf.pos_out[b].cpu().numpy() == ref["pos_out"]).all()
        return out
    if not same_kept:
        r = ref["score"]
        r_k = np.sort(r)[::-1][k - 1]
        diff = np.setxor1d(kept, ref["kept"])
        assert (np.abs(r[diff] - r_k) / r_k).max() < TIE_REL, "kept set differs beyond ties"
        out["close_calls"].append("kept-set tie")
        return out
    # same kept set, different plan: look for the close call in the oracle's fp64 numbers
    X = synth.to_f64(inp["hidden"][b], cfg.h_dtype)[P:P + V]
    C = O.cosine_matrix(X[kept], X[kept])
    sh = ref["s_hat"][kept]
    np.fill_diagonal(C, -np.inf)
    near_t = np.abs(C - threshold) < ROUTE_GAP
    if near_t.any():
        out["close_calls"].append("cosine at the threshold")
    above = C > threshold - ROUTE_GAP
    gap = np.abs(sh[:, None] - sh[None, :])
    ulp = np.spacing(np.maximum(sh[:, None], sh[None, :]).astype(np.float32)).astype(np.float64)
    if (above & (gap < ulp) & (gap > 0)).any():
        out["close_calls"].append("saliences within one f32 unit")
    stronger = (sh[:, None] > sh[None, :]) | ((sh[:, None] == sh[None, :]) &
                                               (np.arange(k)[:, None] < np.arange(k)[None, :]))   # [dest, src]
    Cm = np.where(stronger & (C > threshold), C, -np.inf)
    top2 = np.sort(Cm, axis=0)[-2:]
    if (np.isfinite(top2[0]) & (top2[1] - top2[0] < ROUTE_GAP)).any():
        out["close_calls"].append("two destinations within 1e-5")
    a = k - np.isin(ref["final_idx"], kept).sum()
    pr = ref["pruned"]
    order = pr[np.lexsort((pr, -ref["s_raw"][pr]))]
    if 0 < a < order.size:
        s64 = ref["s_raw"]
        if s64[order[a - 1]] - s64[order[a]] <= 2 * mass_error_bound(inp, b, s64)[[order[a - 1], order[a]]].max():
            out["close_calls"].append("refill boundary within the error of s_raw")
    assert out["close_calls"], "final list or sources differ from the fp64 oracle with no close call to explain it"
    return out


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
        compare_image(inp, buf, b, ref, mu=mu, threshold=thr, report=report, lam_max=lam,
                      eps_=float(np.float32(eps)), mask_on=mask_on)
    return inp, stage
