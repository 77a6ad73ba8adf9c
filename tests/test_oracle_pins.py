"""Pins of the fp64 oracle against what the paper and the mathematics fix.

None of these tests touches the GPU path.  Each pin is chosen so that a plausible
slip in the oracle (dropped term, wrong sign or index, transposed operand, wrong
head mapping, wrong tie rule) fails at least one of them.
"""
import itertools
import math
import os

import numpy as np
import pytest
import scipy.special

from oracle import asap_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.default_rng(seed)


def tiny_qk(seed, H=4, Hkv=2, N=14, d=8):
    r = rng(seed)
    return r.standard_normal((H, N, d)), r.standard_normal((Hkv, N, d))


# ------------------------------------------------------------------ Eq. 2
def test_attention_mass_matches_scalar_triple_loop():
    # Eq. 2 written as scalar sums: s_j = (1/H) sum_h sum_i sum_c q[h,i,c] k[g(h),j,c] / sqrt(d)
    H, Hkv, V, d = 4, 2, 7, 6
    r = rng(0)
    Q = r.standard_normal((H, V, d))
    K = r.standard_normal((Hkv, V, d))
    want = np.zeros(V)
    for j in range(V):
        acc = 0.0
        for h in range(H):
            g = h // (H // Hkv)
            for i in range(V):
                for c in range(d):
                    acc += Q[h, i, c] * K[g, j, c]
        want[j] = acc / math.sqrt(d) / H
    np.testing.assert_allclose(O.attention_mass(Q, K), want, rtol=1e-12, atol=1e-13)


def test_attention_mass_is_a_column_sum_not_a_row_sum():
    # one query row is made huge: every key's mass changes; one key row huge: only that key's
    r = rng(1)
    Q = r.standard_normal((2, 5, 4))
    K = r.standard_normal((2, 5, 4))
    base = O.attention_mass(Q, K)
    K2 = K.copy()
    K2[:, 3] *= 100.0
    s2 = O.attention_mass(Q, K2)
    np.testing.assert_allclose(np.delete(s2, 3), np.delete(base, 3), rtol=1e-12)
    assert abs(s2[3]) > 50 * abs(base[3])


@pytest.mark.parametrize("V,H,Hkv,d", [(16, 4, 4, 8), (96, 6, 2, 16), (576, 4, 2, 32)])
def test_attention_mass_linear_identity(V, H, Hkv, d):
    r = rng(V)
    Q = r.standard_normal((H, V, d))
    K = r.standard_normal((Hkv, V, d))
    a = O.attention_mass(Q, K)
    b = O.attention_mass_linear(Q, K)
    np.testing.assert_allclose(a, b, rtol=1e-10, atol=1e-10 * np.abs(a).max())


def test_gqa_head_mapping():
    # 6 query heads on 3 kv heads: consecutive pairs share a kv head
    assert [O.kv_head(h, 6, 3) for h in range(6)] == [0, 0, 1, 1, 2, 2]
    assert [O.kv_head(h, 28, 4) for h in (0, 6, 7, 13, 14, 27)] == [0, 0, 1, 1, 2, 3]
    assert [O.kv_head(h, 4, 4) for h in range(4)] == [0, 1, 2, 3]


# ------------------------------------------------------------------ Eq. 3
def test_salience_worked_example():
    # s = (1, 3, 2): min 1, max 3 -> (0, 2, 1) / (2 + 1e-6)
    got = O.salience(np.array([1.0, 3.0, 2.0]))
    np.testing.assert_allclose(got, np.array([0.0, 2.0, 1.0]) / (2.0 + 1e-6), rtol=1e-15)


def test_salience_range_and_affine_invariance():
    s = rng(2).standard_normal(100) * 37.0 - 500.0       # "deeply negative" logits
    sh = O.salience(s)
    assert sh.min() == 0.0 and sh[np.argmin(s)] == 0.0
    R = s.max() - s.min()
    assert sh[np.argmax(s)] == pytest.approx(R / (R + 1e-6), rel=1e-15)
    assert sh.max() < 1.0
    # shift invariance is exact up to rounding; positive scaling only moves the eps term
    np.testing.assert_allclose(O.salience(s + 123.0), sh, rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(O.salience(3.0 * s), sh * (R + 1e-6) / (R + 1e-6 / 3.0), rtol=1e-12)
    # order preserving
    assert (np.argsort(sh, kind="stable") == np.argsort(s, kind="stable")).all()


def test_salience_constant_input_is_zero():
    assert (O.salience(np.full(9, -4.25)) == 0.0).all()


# ------------------------------------------------------------------ Eq. 4
def test_mask_log_discount_values():
    sh = np.array([0.0, 1e-9, 0.25, 1.0])
    got = O.mask_log_discount(sh, lambda_max=0.5, eps=1e-6)
    want = np.array([math.log(1e-6), math.log(1e-6), math.log(0.125), math.log(0.5)])
    np.testing.assert_allclose(got, want, rtol=1e-15)
    assert (O.mask_log_discount(sh, mask_on=False) == 0.0).all()


# ------------------------------------------------------------------ Eq. 5
def test_exponent_rule_product_form():
    # exp(W + ln lambda) = lambda exp(W): the log-space mask equals a multiplicative discount
    H, Hkv, V, T, d = 4, 2, 11, 5, 8
    r = rng(3)
    Qt = r.standard_normal((H, T, d))
    Kv = r.standard_normal((Hkv, V, d))
    lam = r.uniform(0.0, 1.0, V)
    lam[2] = 0.0                                     # clamped to eps
    bias = O.mask_log_discount(lam, 1.0, 1e-6)
    A = O.text_visual_attention(Qt, Kv, bias, T)
    lam_c = np.maximum(lam, 1e-6)
    for h in range(H):
        g = h // 2
        for t in range(T):
            w = np.array([lam_c[j] * math.exp(Qt[h, t] @ Kv[g, j] / math.sqrt(d)) for j in range(V)])
            np.testing.assert_allclose(A[h, t], w / w.sum(), rtol=1e-12)


def test_mask_off_is_library_softmax():
    H, Hkv, V, T, d = 3, 3, 17, 4, 16
    r = rng(4)
    Qt = r.standard_normal((H, T + 2, d))            # two padded rows that must be ignored
    Kv = r.standard_normal((Hkv, V, d))
    A = O.text_visual_attention(Qt, Kv, np.zeros(V), T)
    assert A.shape == (H, T, V)
    for h in range(H):
        want = scipy.special.softmax(Qt[h, :T] @ Kv[h].T / math.sqrt(d), axis=1)
        np.testing.assert_allclose(A[h], want, rtol=1e-12)


def test_rows_are_distributions_and_score_sums_to_one():
    H, Hkv, V, T, d = 4, 1, 23, 6, 8
    r = rng(5)
    Qt = r.standard_normal((H, T, d)) * 3.0
    Kv = r.standard_normal((Hkv, V, d)) * 3.0
    bias = O.mask_log_discount(r.uniform(0, 1, V))
    A = O.text_visual_attention(Qt, Kv, bias, T)
    np.testing.assert_allclose(A.sum(axis=2), 1.0, rtol=1e-12)
    assert O.selection_score(A).sum() == pytest.approx(1.0, rel=1e-12)
    lse = r.standard_normal((H, T))
    A2 = O.text_visual_attention(Qt, Kv, bias, T, lse_extra=lse)
    assert (A2.sum(axis=2) < 1.0).all()
    assert O.selection_score(A2).sum() < 1.0


def test_selection_score_is_mean_over_heads_and_rows():
    A = rng(6).uniform(size=(3, 5, 7))
    want = np.zeros(7)
    for h in range(3):
        for t in range(5):
            want += A[h, t]
    np.testing.assert_allclose(O.selection_score(A), want / 15.0, rtol=1e-14)


@pytest.mark.parametrize("P,V,T", [(2, 6, 3), (0, 7, 2), (3, 5, 4)])
def test_text_rows_against_full_nxn_attention(P, V, T):
    """Brute force: full N x N logits, literal mask, full-row softmax.

    (a) The literal Eq. 4 mask is zero on text-query rows, so their attention equals the
        causal (Eq. 1) one.  (b) With lse_extra = log-sum-exp over the row's non-visual
        causal keys, text_visual_attention reproduces the visual columns of those rows.
    (c) Without lse_extra it equals those columns renormalised over the image span."""
    H, Hkv, d = 4, 2, 8
    N = P + V + T
    Q, K = tiny_qk(10 + P, H, Hkv, N, d)
    A_bi, s_hat = O.full_bidirectional_attention(Q, K, P, V, lambda_max=0.7)
    A_ca, _ = O.full_bidirectional_attention(Q, K, P, V, mask="causal")
    text = slice(P + V, N)
    np.testing.assert_allclose(A_bi[:, text], A_ca[:, text], rtol=1e-13)        # (a)
    # visual rows DO change (the mask leaks future keys), and stay distributions
    assert np.abs(A_bi[:, P:P + V] - A_ca[:, P:P + V]).max() > 1e-3
    np.testing.assert_allclose(A_bi.sum(axis=2), 1.0, rtol=1e-12)
    # upper triangle inside the image span carries lambda_j exp(W_ij) weights
    h, i, j = 1, P + 1, P + V - 1
    g = O.kv_head(h, H, Hkv)
    w_ij = math.exp(Q[h, i] @ K[g, j] / math.sqrt(d))
    w_ii = math.exp(Q[h, i] @ K[g, i] / math.sqrt(d))
    lam_j = max(0.7 * s_hat[j - P], 1e-6)
    assert A_bi[h, i, j] / A_bi[h, i, i] == pytest.approx(lam_j * w_ij / w_ii, rel=1e-12)
    # (b)
    lse = np.zeros((H, T))
    for hh in range(H):
        gg = O.kv_head(hh, H, Hkv)
        for t in range(T):
            n_keys = [n for n in range(N) if n <= P + V + t and not (P <= n < P + V)]
            z = np.array([Q[hh, P + V + t] @ K[gg, n] / math.sqrt(d) for n in n_keys])
            lse[hh, t] = scipy.special.logsumexp(z)
    A_t = O.text_visual_attention(Q[:, P + V:], K[:, P:P + V], np.zeros(V), T, lse_extra=lse)
    np.testing.assert_allclose(A_t, A_ca[:, text, P:P + V], rtol=1e-11)
    # (c)
    A_r = O.text_visual_attention(Q[:, P + V:], K[:, P:P + V], np.zeros(V), T)
    ref = A_ca[:, text, P:P + V]
    np.testing.assert_allclose(A_r, ref / ref.sum(axis=2, keepdims=True), rtol=1e-11)


def test_last_token_score_is_the_last_text_row_of_the_full_attention():
    """score_rows="last": the ranking is the last valid text row of the full N x N attention
    (brute force), renormalised over the image span and averaged over heads -- not the mean over
    all text rows, and not a padded row."""
    H, Hkv, d, P, V, T, text_len, D = 4, 2, 8, 2, 9, 4, 3, 6
    N = P + V + T
    Q, K = tiny_qk(31, H, Hkv, N, d)
    X = np.random.default_rng(5).normal(size=(N, D))
    out = O.stage(Q, K, X, text_len, P, V, T, k=4, mask_on=False, mu=0.0, score_rows="last")
    A, _ = O.full_bidirectional_attention(Q, K, P, V, mask="causal")
    row = A[:, P + V + text_len - 1, P:P + V]
    r = (row / row.sum(axis=1, keepdims=True)).mean(axis=0)
    np.testing.assert_allclose(out["score"], r, rtol=1e-11)
    assert out["score"].sum() == pytest.approx(1.0, rel=1e-12)
    every = O.stage(Q, K, X, text_len, P, V, T, k=4, mask_on=False, mu=0.0)
    assert np.abs(every["score"] - out["score"]).max() > 1e-3
    assert set(out["kept"]) == set(np.argsort(-r, kind="stable")[:4])


def test_causal_reference_is_causal():
    Q, K = tiny_qk(20, 2, 2, 9, 4)
    A, _ = O.full_bidirectional_attention(Q, K, 2, 4, mask="causal")
    for i in range(9):
        assert (A[:, i, i + 1:] == 0.0).all()
        np.testing.assert_allclose(A[:, i, :i + 1].sum(axis=1), 1.0, rtol=1e-13)


# ------------------------------------------------------------------ top-k
@pytest.mark.parametrize("seed", range(6))
def test_topk_maximises_sum_over_all_subsets(seed):
    V, k = 9, 4
    r = rng(seed).uniform(size=V)
    kept, pruned = O.select_topk(r, k)
    best = max(itertools.combinations(range(V), k), key=lambda c: r[list(c)].sum())
    assert kept.tolist() == sorted(best)
    assert sorted(kept.tolist() + pruned.tolist()) == list(range(V))
    assert (np.diff(kept) > 0).all() and (np.diff(pruned) > 0).all()


def test_topk_ties_go_to_smaller_index():
    r = np.array([0.5, 0.9, 0.5, 0.5, 0.1, 0.9])
    kept, pruned = O.select_topk(r, 3)
    assert kept.tolist() == [0, 1, 5]
    assert pruned.tolist() == [2, 3, 4]
    kept, _ = O.select_topk(np.zeros(6), 2)
    assert kept.tolist() == [0, 1]
    kept, pruned = O.select_topk(r, 6)
    assert kept.tolist() == list(range(6)) and pruned.size == 0


def test_topk_equals_stable_argsort():
    r = np.round(rng(7).uniform(size=200), 2)        # many ties
    for k in (1, 17, 199):
        kept, _ = O.select_topk(r, k)
        want = np.sort(np.argsort(-r, kind="stable")[:k])
        assert kept.tolist() == want.tolist()


# ------------------------------------------------------------------ similarity routing
def test_route_absorb_double_loop_and_scale_invariance():
    V, D, k = 20, 12, 6
    r = rng(8)
    X = r.standard_normal((V, D))
    kept = np.array([1, 4, 5, 11, 12, 19])
    pruned = np.array([j for j in range(V) if j not in kept])
    assign, best = O.route_absorb(X, kept, pruned)
    for a, j in enumerate(pruned):
        cs = [X[j] @ X[i] / (np.linalg.norm(X[j]) * np.linalg.norm(X[i])) for i in kept]
        assert assign[a] == int(np.argmax(cs))
        assert best[a] == pytest.approx(max(cs), rel=1e-12)
    assert (np.abs(best) <= 1.0 + 1e-12).all()
    Xs = X.copy()
    Xs[::3] *= 8.0                                   # high-norm outlier tokens
    assign2, best2 = O.route_absorb(Xs, kept, pruned)
    assert (assign2 == assign).all()
    np.testing.assert_allclose(best2, best, rtol=1e-12)


def test_route_absorb_tie_and_threshold():
    X = np.array([[1.0, 0.0], [1.0, 0.0], [0.0, 1.0], [2.0, 0.0], [1.0, 1.0]])
    kept = np.array([0, 1, 2])
    pruned = np.array([3, 4])
    assign, best = O.route_absorb(X, kept, pruned)
    assert assign.tolist() == [0, 0]                 # token 3 ties between 0 and 1 -> 0
    np.testing.assert_allclose(best, [1.0, math.sqrt(0.5)], rtol=1e-15)
    assign, _ = O.route_absorb(X, kept, pruned, threshold=0.9)
    assert assign.tolist() == [0, -1]


def test_cosine_norm_floor():
    X = np.array([[0.0, 0.0], [3.0, 4.0]])
    C = O.cosine_matrix(X, X)
    assert C[0, 0] == 0.0 and C[0, 1] == 0.0 and C[1, 1] == pytest.approx(1.0)


# ------------------------------------------------------------------ Eq. 6
def merge_case(seed, V=30, D=16, k=8):
    r = rng(seed)
    X = r.standard_normal((V, D))
    s_hat = r.uniform(size=V)
    s_hat[r.integers(V)] = 0.0
    kept = np.sort(r.choice(V, k, replace=False))
    pruned = np.array([j for j in range(V) if j not in kept])
    assign = r.integers(-1, k, size=pruned.size)
    return X, s_hat, kept, pruned, assign


@pytest.mark.parametrize("mu", [1.0, 0.5])
def test_merge_conservation_laws(mu):
    X, s_hat, kept, pruned, assign = merge_case(9)
    k = kept.size
    y, wsum = O.weighted_merge(X, s_hat, kept, O.sources_from_assign(assign, pruned, k), mu)
    members = pruned[assign >= 0]
    assert wsum.sum() == pytest.approx(s_hat[kept].sum() + mu * s_hat[members].sum(), rel=1e-13)
    lhs = (wsum[:, None] * y).sum(axis=0)
    rhs = (s_hat[kept, None] * X[kept]).sum(axis=0) + mu * (s_hat[members, None] * X[members]).sum(axis=0)
    np.testing.assert_allclose(lhs, rhs, rtol=1e-12, atol=1e-12)
    for c in range(k):                               # convex combination: inside the hull
        grp = np.concatenate([[kept[c]], pruned[assign == c]])
        assert (y[c] <= X[grp].max(axis=0) + 1e-12).all()
        assert (y[c] >= X[grp].min(axis=0) - 1e-12).all()


def test_merge_worked_example():
    # Eq. 6 by hand: destination weight 0.5 with value 2, sources 0.25 -> 6 and 0.25 -> 10
    X = np.array([[2.0], [6.0], [10.0], [100.0]])
    s_hat = np.array([0.5, 0.25, 0.25, 0.9])
    y, w = O.weighted_merge(X, s_hat, np.array([0]), [np.array([1, 2])])
    assert y[0, 0] == pytest.approx((0.5 * 2 + 0.25 * 6 + 0.25 * 10) / 1.0)
    assert w[0] == pytest.approx(1.0)


def test_merge_weight_zero_and_zero_denominator():
    X, s_hat, kept, pruned, assign = merge_case(10)
    k = kept.size
    y, wsum = O.weighted_merge(X, s_hat, kept, O.sources_from_assign(assign, pruned, k), 0.0)
    nz = s_hat[kept] > 0
    np.testing.assert_allclose(y[nz], X[kept][nz], rtol=1e-15)
    np.testing.assert_allclose(wsum, s_hat[kept])
    s0 = np.zeros_like(s_hat)
    y0, w0 = O.weighted_merge(X, s0, kept, O.sources_from_assign(assign, pruned, k), 1.0)
    assert (y0 == X[kept]).all() and (w0 == 0.0).all()


# ------------------------------------------------------------------ paper routing + salvage
@pytest.mark.parametrize("seed", range(4))
def test_route_paper_structure(seed):
    r = rng(30 + seed)
    V, D, k = 60, 24, 20
    centres = r.standard_normal((5, D))
    X = centres[r.integers(5, size=V)] + 0.2 * r.standard_normal((V, D))
    s_raw = r.standard_normal(V) * 10
    s_hat = O.salience(s_raw)
    kept, pruned = O.select_topk(r.uniform(size=V), k)
    final_idx, sources = O.route_paper(X, s_raw, s_hat, kept, pruned, threshold=0.8)
    assert final_idx.size == k and (np.diff(final_idx) > 0).all()       # exactly k survivors
    all_src = np.concatenate([s for s in sources]) if sources else np.zeros(0, int)
    assert len(set(all_src.tolist())) == all_src.size                   # disjoint source sets
    assert set(all_src.tolist()).issubset(set(kept.tolist()))
    assert not set(all_src.tolist()) & set(final_idx.tolist())           # roots are never sources
    a = all_src.size
    salvaged = sorted(set(final_idx.tolist()) - set(kept.tolist()))
    assert len(salvaged) == a
    want = pruned[np.lexsort((pruned, -s_raw[pruned]))[:a]]
    assert salvaged == sorted(want.tolist())                            # top-a by raw mass
    for c, i in enumerate(final_idx):
        for j in sources[c]:                                            # flows toward higher salience
            assert (s_hat[i], -i) > (s_hat[j], -j)
        if i in salvaged:
            assert sources[c].size == 0
    assert a > 0                                                        # the case does merge


def test_route_paper_threshold_one_is_plain_topk():
    r = rng(40)
    X = r.standard_normal((25, 8))
    s_raw = r.standard_normal(25)
    kept, pruned = O.select_topk(r.uniform(size=25), 7)
    final_idx, sources = O.route_paper(X, s_raw, O.salience(s_raw), kept, pruned, threshold=1.0)
    assert (final_idx == kept).all() and all(s.size == 0 for s in sources)


def test_route_paper_chain_resolves_to_root():
    # three collinear tokens with increasing salience: 0 -> (1 or 2), 1 -> 2; all end in 2
    X = np.array([[1.0, 0.0], [1.0, 0.01], [1.0, 0.02], [0.0, 1.0], [0.0, -1.0]])
    s_raw = np.array([1.0, 2.0, 3.0, 0.5, 0.4])
    s_hat = O.salience(s_raw)
    kept = np.array([0, 1, 2])
    pruned = np.array([3, 4])
    final_idx, sources = O.route_paper(X, s_raw, s_hat, kept, pruned, threshold=0.9)
    assert final_idx.tolist() == [2, 3, 4]
    assert sources[0].tolist() == [0, 1] and sources[1].size == 0 and sources[2].size == 0


def _unit(deg):
    return [math.cos(math.radians(deg)), math.sin(math.radians(deg))]


@pytest.mark.parametrize("order", ["far_first", "near_first"])
def test_route_paper_takes_the_most_similar_of_two_eligible_roots(order):
    """Sec. 4.2, several eligible destinations for one source.  Three kept tokens in the plane:
    the source j at 0 degrees, one stronger token at +30 degrees (cosine 0.866 to j), another at
    -20 degrees (cosine 0.940).  The two stronger tokens are 50 degrees apart (cosine 0.643 < t =
    0.8), so neither merges into the other: they are roots of different trees and j has to choose.
    The nearer one (-20 degrees) must absorb it, wherever it stands in the index order."""
    far, near, src = _unit(30.0), _unit(-20.0), _unit(0.0)
    filler = [[0.0, 0.0, 1.0], [0.0, 0.0, -1.0]]                 # pruned tokens, orthogonal to the plane
    if order == "far_first":
        X = np.array([far + [0.0], near + [0.0], src + [0.0]] + filler)
        i_far, i_near, i_src = 0, 1, 2
    else:
        X = np.array([near + [0.0], far + [0.0], src + [0.0]] + filler)
        i_near, i_far, i_src = 0, 1, 2
    s_raw = np.zeros(5)
    s_raw[i_far], s_raw[i_near], s_raw[i_src] = 5.0, 4.0, 1.0    # both stronger than the source
    s_raw[3], s_raw[4] = 0.7, 0.2
    s_hat = O.salience(s_raw)
    kept, pruned = np.array([0, 1, 2]), np.array([3, 4])
    final_idx, sources = O.route_paper(X, s_raw, s_hat, kept, pruned, threshold=0.8)
    # one slot is vacated and refilled with the pruned token of larger raw mass (token 3)
    assert final_idx.tolist() == [0, 1, 3]
    got = {int(i): s.tolist() for i, s in zip(final_idx, sources)}
    assert got[i_near] == [i_src] and got[i_far] == [] and got[3] == []


def test_route_paper_equal_salience_goes_to_the_smaller_index():
    """Sec. 4.2: ties in salience are broken by sequence index.  Tokens 1 and 2 are near-duplicates
    (cosine 0.99995 > t) with bit-equal salience; the one that comes first in the sequence is the
    anchor, so token 1 absorbs token 2 and not the other way round.  Token 0 is unrelated."""
    X = np.array([[0.0, 1.0, 0.0], [1.0, 0.0, 0.0], [1.0, 0.01, 0.0], [0.0, 0.0, 1.0], [0.0, 0.0, -1.0]])
    s_raw = np.array([3.0, 2.0, 2.0, 0.5, 1.5])
    s_hat = O.salience(s_raw)
    assert s_hat[1] == s_hat[2]
    kept, pruned = np.array([0, 1, 2]), np.array([3, 4])
    final_idx, sources = O.route_paper(X, s_raw, s_hat, kept, pruned, threshold=0.9)
    assert final_idx.tolist() == [0, 1, 4]                       # token 2 left; refill = largest raw mass
    assert [s.tolist() for s in sources] == [[], [2], []]


def test_stage_merge_weights_are_the_saliences_not_the_raw_masses():
    """Whole stage with mu = 1 on a case small enough to do by hand (Eq. 2, 3, 6).  One head of size
    1, three visual tokens, one text token, budget 1.  Visual queries 0.5, 0.25, 0.25 sum to 1 and
    the keys are 1, 3, 2, so Eq. 2 gives the raw masses s = (1, 3, 2) and Eq. 3 the saliences
    s_hat = (0, 2, 1) / (2 + eps).  The text query 1 sees logits 1, 3, 2 plus the log-discounts, so
    token 1 is kept and absorbs tokens 0 and 2 (no threshold).  Eq. 6 weighs with s_hat: hidden
    states 10, 20, 40 give (2*20 + 1*40 + 0*10) / 3 = 80/3; weighing with the raw masses instead
    would give (3*20 + 2*40 + 1*10) / 6 = 25."""
    P, V, T, k = 0, 3, 1, 1
    Q = np.array([[[0.5], [0.25], [0.25], [1.0]]])               # [H=1, N=4, d=1]
    K = np.array([[[1.0], [3.0], [2.0], [0.0]]])
    X = np.array([[10.0, -1.0], [20.0, 2.0], [40.0, 4.0], [7.0, 7.0]])
    out = O.stage(Q, K, X, T, P, V, T, k, mu=1.0)
    np.testing.assert_allclose(out["s_raw"], [1.0, 3.0, 2.0], rtol=1e-15)
    np.testing.assert_allclose(out["s_hat"], np.array([0.0, 2.0, 1.0]) / (2.0 + 1e-6), rtol=1e-15)
    assert out["kept"].tolist() == [1] and out["pruned"].tolist() == [0, 2]
    assert out["assign"].tolist() == [0, 0]
    np.testing.assert_allclose(out["y"][0], [80.0 / 3.0, (2 * 2.0 + 1 * 4.0) / 3.0], rtol=1e-14)
    np.testing.assert_allclose(out["wsum"], [3.0 / (2.0 + 1e-6)], rtol=1e-15)
    assert abs(out["y"][0, 0] - 25.0) > 1.0                      # not the raw-mass weighting
    np.testing.assert_allclose(out["Y"][:out["new_len"]], [out["y"][0], X[3]], rtol=1e-14)
    # the paper's routing uses the same Eq. 6 weights: kept = {1, 2} (cosine 1 > t), 2 -> 1, refill 0
    X2 = np.array([[10.0, -1.0], [20.0, 2.0], [40.0, 4.0], [7.0, 7.0]])
    out2 = O.stage(Q, K, X2, T, P, V, T, 2, mu=1.0, route="paper", threshold=0.99)
    assert out2["kept"].tolist() == [1, 2] and out2["final_idx"].tolist() == [0, 1]
    np.testing.assert_allclose(out2["y"], [X2[0], (2 * X2[1] + 1 * X2[2]) / 3.0], rtol=1e-14)


# ------------------------------------------------------------------ sequence assembly, K/V
def test_assemble_and_gather():
    P, V, Tmax, tl = 2, 6, 3, 2
    N = P + V + Tmax
    X = np.arange(N * 2, dtype=np.float64).reshape(N, 2)
    final_idx = np.array([1, 4])
    y = np.array([[-1.0, -1.0], [-2.0, -2.0]])
    Y, pos, new_len = O.assemble_sequence(X, y, final_idx, P, V, Tmax, tl)
    assert new_len == 6
    assert pos.tolist() == [0, 1, 3, 6, 8, 9, -1]
    assert (Y[:2] == X[:2]).all() and (Y[2:4] == y).all() and (Y[4:6] == X[8:10]).all()
    cache = rng(50).standard_normal((3, N, 4))
    got = O.gather_kv(cache, pos, new_len)
    assert got.shape == (3, 6, 4)
    for n in range(6):
        assert (got[:, n] == cache[:, pos[n]]).all()


def test_paged_gather_against_hand_placed_tokens():
    """Paged K/V gather.  Token values encode (token, head) so every placement can be read off by
    hand: a 7-token sequence scattered over pages 5, 0, 3 of a pool with 3 slots per page is
    compacted to tokens 0, 2, 3, 6 in pages 4, 1.  Every other slot of the destination pool keeps
    its sentinel, and with pages laid out in order the result is the contiguous gather."""
    Hkv, d, ps = 2, 3, 3
    src_pages, dst_pages = np.array([5, 0, 3]), np.array([4, 1])
    src_pool = np.full((6, Hkv, ps, d), -7.0)
    for n in range(7):
        for g in range(Hkv):
            src_pool[src_pages[n // ps], g, n % ps] = 100 * n + 10 * g + np.arange(d)
    pos, new_len = np.array([0, 2, 3, 6, -1, -1]), 4
    dst_pool = np.full((6, Hkv, ps, d), -1.0)
    O.gather_kv_paged(src_pool, src_pages, dst_pool, dst_pages, pos, new_len)
    expect = np.full((6, Hkv, ps, d), -1.0)
    for g in range(Hkv):
        expect[4, g, 0] = 0 + 10 * g + np.arange(d)       # token 0 -> page 4 slot 0
        expect[4, g, 1] = 200 + 10 * g + np.arange(d)     # token 2 -> page 4 slot 1
        expect[4, g, 2] = 300 + 10 * g + np.arange(d)     # token 3 -> page 4 slot 2
        expect[1, g, 0] = 600 + 10 * g + np.arange(d)     # token 6 -> page 1 slot 0
    assert (dst_pool == expect).all()
    # identity tables: the pool is the contiguous cache cut into pages
    N, ps2 = 12, 4
    cache = rng(51).standard_normal((Hkv, N, d))
    pool = cache.reshape(Hkv, N // ps2, ps2, d).transpose(1, 0, 2, 3).copy()
    pos2, nl2 = np.array([1, 2, 5, 7, 8, 11, -1, -1]), 6
    out_pool = np.zeros((2, Hkv, ps2, d))
    O.gather_kv_paged(pool, np.arange(3), out_pool, np.arange(2), pos2, nl2)
    flat = out_pool.transpose(1, 0, 2, 3).reshape(Hkv, 8, d)
    assert (flat[:, :nl2] == cache[:, pos2[:nl2]]).all() and (flat[:, nl2:] == 0).all()


# ------------------------------------------------------------------ whole stage: reduction invariant
def test_stage_reduces_to_plain_topk_attention_pruning():
    """Mask off and merge weight 0 => the stage is the baseline the ablation starts from:
    keep the k visual tokens that receive the most text attention (computed here from the
    brute-force causal N x N attention), hidden rows copied unchanged."""
    H, Hkv, d, D, P, V, T, k = 4, 2, 8, 10, 2, 12, 3, 5
    N = P + V + T
    r = rng(60)
    Q = r.standard_normal((H, N, d))
    K = r.standard_normal((Hkv, N, d))
    X = r.standard_normal((N, D))
    out = O.stage(Q, K, X, T, P, V, T, k, mask_on=False, mu=0.0)
    A, _ = O.full_bidirectional_attention(Q, K, P, V, mask="causal")
    vis = A[:, P + V:, P:P + V]
    vis = vis / vis.sum(axis=2, keepdims=True)
    recv = vis.mean(axis=(0, 1))
    want = np.sort(np.argsort(-recv, kind="stable")[:k])
    assert out["kept"].tolist() == want.tolist()
    assert (out["Y"][:P] == X[:P]).all()
    assert (out["Y"][P:P + k] == X[P + want]).all()
    assert (out["Y"][P + k:P + k + T] == X[P + V:]).all()
    assert out["pos_out"][:out["new_len"]].tolist() == list(range(P)) + (P + want).tolist() + \
        list(range(P + V, N))
    # with the mask on the kept set differs for this seed (the discount matters)
    out_m = O.stage(Q, K, X, T, P, V, T, k, mask_on=True, mu=0.0)
    assert out_m["kept"].tolist() != want.tolist()
    assert (out_m["Y"][P:P + k] == X[P + out_m["kept"]]).all()


def test_stage_lambda_max_cancels_over_visual_span():
    # over the visual span alone a uniform factor lambda_max cancels unless the eps clamp bites
    H, Hkv, d, D, P, V, T, k = 2, 2, 8, 6, 1, 10, 2, 4
    r = rng(61)
    N = P + V + T
    Q, K, X = r.standard_normal((H, N, d)), r.standard_normal((Hkv, N, d)), r.standard_normal((N, D))
    a = O.stage(Q, K, X, T, P, V, T, k, lambda_max=1.0, eps=1e-30)
    b = O.stage(Q, K, X, T, P, V, T, k, lambda_max=0.3, eps=1e-30)
    j0 = int(np.argmin(a["s_hat"]))                  # lambda = eps there: the clamp bites
    np.testing.assert_allclose(np.delete(a["score"], j0), np.delete(b["score"], j0), rtol=1e-10)
    assert a["score"][j0] < 1e-20


def test_stage_linear_mass_flag_matches():
    H, Hkv, d, D, P, V, T, k = 4, 2, 16, 12, 3, 40, 5, 9
    r = rng(62)
    N = P + V + T
    Q, K, X = r.standard_normal((H, N, d)), r.standard_normal((Hkv, N, d)), r.standard_normal((N, D))
    a = O.stage(Q, K, X, 4, P, V, T, k)
    b = O.stage(Q, K, X, 4, P, V, T, k, linear_mass=True)
    assert (a["kept"] == b["kept"]).all()
    np.testing.assert_allclose(a["Y"], b["Y"], rtol=1e-9, atol=1e-12)
    assert a["new_len"] == P + k + 4


# ------------------------------------------------------------------ Eq. 7 / Eq. 8 printed values
def read_table(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                rows.append(line.split())
    return rows


def test_flops_formula_against_printed_tables():
    for row in read_table("eq7_flops.txt"):
        v, printed = int(row[0]), float(row[1])
        got = O.theoretical_flops([32], [v], 4096, 11008) / 1e12
        assert abs(got - printed) <= 0.0006, (v, got, printed)       # printed to 3 decimals


def test_flops_ratio_against_printed_table():
    for row in read_table("eq8_ratio.txt"):
        v, v0, pct = int(row[0]), int(row[1]), float(row[2])
        assert abs(100.0 * O.flops_ratio([32], [v], v0, 4096, 11008) - pct) <= 0.006


def test_flops_multi_stage_sum():
    d, m = 64, 128
    want = 2 * O.layer_flops(100, d, m) + 3 * O.layer_flops(40, d, m) + 5 * O.layer_flops(10, d, m)
    assert O.theoretical_flops([2, 3, 5], [100, 40, 10], d, m) == want
    assert O.layer_flops(3, 5, 7) == 4 * 3 * 25 + 2 * 9 * 5 + 3 * 3 * 5 * 7


# ---------------------------------------------------------------- attention forward under the Eq. 4-5 mask
def _small_qkv(seed, H=2, Hkv=1, N=9, d=4):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((H, N, d)), rng.standard_normal((Hkv, N, d)), rng.standard_normal((Hkv, N, d)))


def test_attention_forward_rows_are_convex_combinations():
    # every row of A sums to one: constant values come out unchanged, whatever the mask
    Q, K, Vv = _small_qkv(3)
    Vc = np.broadcast_to(np.array([1.5, -2.0, 0.25, 7.0]), Vv.shape).copy()
    for mask in ("bidir", "causal"):
        out, _ = O.attention_forward(Q, K, Vc, 2, 5, lambda_max=0.8, mask=mask)
        assert np.abs(out - Vc[0, 0]).max() < 1e-12


def test_attention_forward_two_token_closed_form():
    # N = 2, causal: row 0 sees key 0 only; row 1 is the two-term softmax written out
    Q, K, Vv = _small_qkv(5, H=1, Hkv=1, N=2, d=3)
    out, _ = O.attention_forward(Q, K, Vv, 0, 1, mask="causal")
    assert np.allclose(out[0, 0], Vv[0, 0], rtol=0, atol=1e-15)
    w0, w1 = Q[0, 1] @ K[0, 0] / math.sqrt(3), Q[0, 1] @ K[0, 1] / math.sqrt(3)
    want = (math.exp(w0) * Vv[0, 0] + math.exp(w1) * Vv[0, 1]) / (math.exp(w0) + math.exp(w1))
    assert np.allclose(out[0, 1], want, rtol=1e-13, atol=1e-15)


def test_attention_forward_mask_touches_only_image_rows_and_adds_discounted_future_keys():
    P, V = 2, 4
    Q, K, Vv = _small_qkv(8, H=2, Hkv=2, N=9, d=4)
    lam = 0.6
    out_bi, s_hat = O.attention_forward(Q, K, Vv, P, V, lambda_max=lam, mask="bidir")
    out_ca, _ = O.attention_forward(Q, K, Vv, P, V, mask="causal")
    rows = np.arange(9)
    outside = (rows < P) | (rows >= P + V - 1)        # the last image row has no future image key
    assert np.array_equal(out_bi[:, outside], out_ca[:, outside])
    assert np.abs(out_bi[:, P:P + V - 1] - out_ca[:, P:P + V - 1]).max() > 1e-6
    # image row i written out: keys <= i with weight e^w, future image keys with weight lam' e^w
    h, i = 1, P + 1
    w = Q[h, i] @ K[h].T / 2.0
    wt = np.zeros(9)
    wt[:i + 1] = np.exp(w[:i + 1])
    for j in range(i + 1, P + V):
        wt[j] = max(lam * s_hat[j - P], 1e-6) * math.exp(w[j])
    want = (wt[:, None] * Vv[h]).sum(0) / wt.sum()
    assert np.allclose(out_bi[h, i], want, rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------- Sec. 3.1: RoPE score, Eq. 2 from hidden states
def test_rope_is_a_rotation_and_the_score_depends_on_the_distance_only():
    """Sec. 3.1: s(m, n) = x_m^T W_q^T R_{m-n} W_k x_n.  Rotations keep norms; position 0 is the
    identity; and the score of a query at m with a key at n is the score at (m - n, 0)."""
    r = rng(70)
    d = 8
    q, k = r.standard_normal((1, d)), r.standard_normal((1, d))
    assert np.allclose(O.rope_rotate(q, [0]), q, rtol=0, atol=0)
    for m, n in ((5, 2), (100, 97), (3, 0), (2300, 35)):
        qm, kn = O.rope_rotate(q, [m]), O.rope_rotate(k, [n])
        assert abs(np.linalg.norm(qm) - np.linalg.norm(q)) < 1e-12
        ref = O.rope_rotate(q, [m - n]) @ k.T
        assert abs((qm @ kn.T - ref).item()) < 1e-10 * (1 + abs(ref.item()))


def test_rope_pairs_and_frequencies_by_hand():
    # d = 4, theta = 100: pairs (0, 2) at frequency 1 and (1, 3) at frequency 100^(-1/2) = 0.1
    v = np.array([[1.0, 2.0, 3.0, 4.0]])
    out = O.rope_rotate(v, [2.0], theta=100.0)[0]
    a0, a1 = 2.0 * 1.0, 2.0 * 0.1
    want = [1.0 * math.cos(a0) - 3.0 * math.sin(a0), 2.0 * math.cos(a1) - 4.0 * math.sin(a1),
            3.0 * math.cos(a0) + 1.0 * math.sin(a0), 4.0 * math.cos(a1) + 2.0 * math.sin(a1)]
    np.testing.assert_allclose(out, want, rtol=1e-14)


def test_mass_from_hidden_states_equals_the_column_sums_of_the_alignment_matrix():
    """Eq. 2 from hidden states: project every visual token (q = R W_q x, Sec. 3.1), build W = Q K^T /
    sqrt(d) and sum its columns (attention_mass, pinned above by the scalar triple loop); the summed
    queries must give the same masses, GQA included, and the head mapping must matter."""
    H, Hkv, d, D, V, P = 4, 2, 8, 12, 9, 3
    r = rng(71)
    X, Wq, K = r.standard_normal((V, D)), r.standard_normal((H * d, D)), r.standard_normal((Hkv, V, d))
    pos = P + np.arange(V)
    Q = O.project_queries(X, Wq, pos, H, d, theta=50.0)
    assert Q.shape == (H, V, d)
    # one token by hand: head 1 of token 2 is the rotation of rows d..2d-1 of W_q times x_2
    np.testing.assert_allclose(Q[1, 2], O.rope_rotate((Wq[d:2 * d] @ X[2])[None, :], [pos[2]], 50.0)[0], rtol=1e-13)
    qbar = O.summed_visual_queries(X, Wq, pos, H, Hkv, d, theta=50.0)
    np.testing.assert_allclose(O.attention_mass_from_summed_queries(qbar, K, H), O.attention_mass(Q, K),
                               rtol=1e-12, atol=1e-13)
    swapped = qbar[::-1]
    assert np.abs(O.attention_mass_from_summed_queries(swapped, K, H) - O.attention_mass(Q, K)).max() > 1e-3
