"""Plain fp64 CPU oracle of the ASAP pruning stage.  TEST INFRASTRUCTURE ONLY.

Only tests/, the smoke check and the benchmark's cpu_baseline leg may import
this file; the product (HIP) path never does, and this file imports nothing
from it.  Every function takes and returns float64 / integer NumPy arrays for
ONE image (images are independent) and follows the paper's steps in the paper's
order and notation, with no blocking, fusion or reordering:

  attention_mass            Eq. 2   s_j = sum_{i in I} W_ij,  W = Q K^T / sqrt(d)   (Sec. 4.1)
  attention_mass_linear     the same sum taken on the query side first (algebraic identity,
                            pinned to attention_mass by test; used at full workload sizes)
  salience                  Eq. 3   min-max normalisation with eps = 1e-6
  mask_log_discount         Eq. 4   ln(max(lambda_max * s_hat_j, eps))
  text_visual_attention     Eq. 5   softmax of text-query rows over the visual keys
  selection_score           mean attention a visual key receives (Fig. 3: "retains top-k")
  select_topk               top-k, ties to the smaller index
  route_absorb              cosine similarity (Sec. 4.2) of each pruned token to each kept token
  route_paper               Sec. 4.2 routing inside the kept set + budget reallocation
  attention_forward         output of one attention layer under the Eq. 4-5 mask (whole sequence)
  weighted_merge            Eq. 6
  assemble_sequence         prefix | merged kept tokens | text           (Fig. 3 caption)
  gather_kv                 K/V rows of surviving positions
  gather_kv_paged           the same for caches kept as pools of pages with block tables
  stage                     all steps for one image (score_rows="last": ranking by the last text token)
  full_bidirectional_attention   literal N x N Eq. 4-5, brute force, for pins only
  theoretical_flops / flops_ratio   Eq. 7 / Eq. 8 (appendix)
  rope_rotate / project_queries / summed_visual_queries / attention_mass_from_summed_queries
                            Sec. 3.1: q_m = R_{Theta,m} W_q x_m, and Eq. 2 taken from the hidden states

Readings taken where the paper is silent (each is listed in the design notes):
heads are averaged (Eq. 2-4 carry no head index); the selection score is the
mean, over heads and valid text rows, of the softmax weight each visual key
gets, with Eq. 4's per-key log-discount added to those rows' logits; the
softmax runs over the visual span unless lse_extra supplies the rest of the row;
ties go to the smaller index; cosine norms are clamped at 1e-8; a zero
denominator in Eq. 6 leaves the token unchanged.

Pins (tests/test_oracle_pins.py): brute-force N x N attention, subset
enumeration for top-k, double-loop cosine, conservation laws of Eq. 6, the
mask-off / no-merge reduction to plain top-k attention pruning, library softmax,
and the six FLOPs values printed in Tables 1, 2 and 5.  Not pinned by anything
(no code, weights or data exist to pin it): that these readings are what the
authors ran -- "parity unpinned" for that question only.
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence, Tuple

import numpy as np

EPS_DEFAULT = 1e-6
NORM_FLOOR = 1e-8


def kv_head(h: int, H: int, Hkv: int) -> int:
    """Key/value head serving query head h under grouped-query attention."""
    return (h * Hkv) // H


# ---------------------------------------------------------------- Eq. 2
def attention_mass(Qv: np.ndarray, Kv: np.ndarray) -> np.ndarray:
    """Eq. 2.  Qv [H,V,d] visual queries, Kv [Hkv,V,d] visual keys -> s [V].

    Builds each head's V x V alignment matrix W = Q K^T / sqrt(d) and sums its
    columns over all visual query rows; heads are averaged."""
    H, V, d = Qv.shape
    Hkv = Kv.shape[0]
    s = np.zeros(V, dtype=np.float64)
    for h in range(H):
        W = (Qv[h] @ Kv[kv_head(h, H, Hkv)].T) / math.sqrt(d)      # W[i, j]
        s += W.sum(axis=0)
    return s / H


def attention_mass_linear(Qv: np.ndarray, Kv: np.ndarray) -> np.ndarray:
    """Eq. 2 with the sum over query rows taken before the product:
    sum_i (q_i . k_j) = (sum_i q_i) . k_j."""
    H, V, d = Qv.shape
    Hkv = Kv.shape[0]
    s = np.zeros(V, dtype=np.float64)
    for h in range(H):
        qbar = Qv[h].sum(axis=0)
        s += (Kv[kv_head(h, H, Hkv)] @ qbar) / math.sqrt(d)
    return s / H


# ---------------------------------------------------------------- Eq. 3
def salience(s: np.ndarray, eps: float = EPS_DEFAULT) -> np.ndarray:
    """Eq. 3: s_hat_j = (s_j - s_min) / (s_max - s_min + eps)."""
    s_min = s.min()
    s_max = s.max()
    return (s - s_min) / (s_max - s_min + eps)


# ---------------------------------------------------------------- Eq. 4
def mask_log_discount(s_hat: np.ndarray, lambda_max: float = 1.0, eps: float = EPS_DEFAULT,
                      mask_on: bool = True) -> np.ndarray:
    """Eq. 4's off-causal entry for key j: ln(max(lambda_j, eps)), lambda_j = lambda_max * s_hat_j.
    With the mask off the discount is ln(1) = 0."""
    if not mask_on:
        return np.zeros_like(s_hat)
    lam = lambda_max * s_hat
    return np.log(np.maximum(lam, eps))


# ---------------------------------------------------------------- Eq. 5 on the text rows
def text_visual_attention(Qt: np.ndarray, Kv: np.ndarray, log_discount: np.ndarray,
                          text_len: int, lse_extra: Optional[np.ndarray] = None) -> np.ndarray:
    """Eq. 5 for text-query rows over visual keys.

    Qt [H,Tmax,d] (rows >= text_len ignored), Kv [Hkv,V,d], log_discount [V] added to
    every row's logits.  lse_extra [H,Tmax], when given, is log(sum exp) of the row's
    logits over its non-visual keys, so that the row is normalised as in the full
    softmax.  Returns A [H, text_len, V]."""
    H, _, d = Qt.shape
    Hkv, V, _ = Kv.shape
    A = np.zeros((H, text_len, V), dtype=np.float64)
    for h in range(H):
        Z = (Qt[h, :text_len] @ Kv[kv_head(h, H, Hkv)].T) / math.sqrt(d) + log_discount[None, :]
        m = Z.max(axis=1)
        if lse_extra is not None:
            m = np.maximum(m, lse_extra[h, :text_len])
        E = np.exp(Z - m[:, None])
        den = E.sum(axis=1)
        if lse_extra is not None:
            den = den + np.exp(lse_extra[h, :text_len] - m)
        A[h] = E / den[:, None]
    return A


def selection_score(A: np.ndarray) -> np.ndarray:
    """r_j = mean over heads and text rows of A[h,t,j]."""
    H, T, _ = A.shape
    return A.sum(axis=(0, 1)) / (H * T)


# ---------------------------------------------------------------- top-k
def select_topk(r: np.ndarray, k: int) -> Tuple[np.ndarray, np.ndarray]:
    """Keep the k largest r_j, ties to the smaller index.  Returns (kept, pruned),
    both ascending, int64."""
    V = r.shape[0]
    order = np.lexsort((np.arange(V), -r))          # primary -r ascending, then index
    kept = np.sort(order[:k])
    mask = np.ones(V, dtype=bool)
    mask[kept] = False
    return kept.astype(np.int64), np.nonzero(mask)[0].astype(np.int64)


# ---------------------------------------------------------------- Sec. 4.2 similarity
def cosine_matrix(Xa: np.ndarray, Xb: np.ndarray) -> np.ndarray:
    """Pairwise cosine similarity of rows of Xa with rows of Xb; norms floored at 1e-8."""
    na = np.maximum(np.sqrt((Xa * Xa).sum(axis=1)), NORM_FLOOR)
    nb = np.maximum(np.sqrt((Xb * Xb).sum(axis=1)), NORM_FLOOR)
    return (Xa @ Xb.T) / (na[:, None] * nb[None, :])


def route_absorb(Xv: np.ndarray, kept: np.ndarray, pruned: np.ndarray,
                 threshold: float = -math.inf) -> Tuple[np.ndarray, np.ndarray]:
    """Each pruned token goes to its most similar kept token (ties: smaller index).

    Xv [V,D].  Returns assign [V-k] = slot in 0..k-1 (position in `kept`) or -1 when the
    best similarity does not exceed `threshold`, and best [V-k] that similarity."""
    if pruned.size == 0:
        return np.zeros(0, dtype=np.int64), np.zeros(0, dtype=np.float64)
    C = cosine_matrix(Xv[pruned], Xv[kept])
    assign = np.argmax(C, axis=1)                    # first maximum = smallest kept index
    best = C[np.arange(C.shape[0]), assign]
    assign = np.where(best > threshold, assign, -1)
    return assign.astype(np.int64), best


def route_paper(Xv: np.ndarray, s_raw: np.ndarray, s_hat: np.ndarray, kept: np.ndarray,
                pruned: np.ndarray, threshold: float):
    """Sec. 4.2: redundancy removal inside the kept set, then budget reallocation.

    A kept token j is a source iff some other kept i has cosine S_ij > threshold and
    (s_hat_i, -i) > (s_hat_j, -j); it goes to the most similar such i (ties: smaller
    index) and chains are followed to their root, so every tree merges into one
    token that is not itself a source.  The a vacated slots are refilled with the a
    pruned tokens of largest raw mass s_j (ties: smaller index), which stay unmerged.

    Returns (final_idx [k] ascending, sources: list of arrays of visual indices absorbed
    by each final token, in final_idx order)."""
    k = kept.size
    C = cosine_matrix(Xv[kept], Xv[kept])
    dest = np.full(k, -1, dtype=np.int64)
    for a in range(k):
        j = kept[a]
        best_c, best_b = -math.inf, -1
        for b in range(k):
            if b == a:
                continue
            i = kept[b]
            stronger = (s_hat[i] > s_hat[j]) or (s_hat[i] == s_hat[j] and i < j)
            if stronger and C[b, a] > threshold and C[b, a] > best_c:
                best_c, best_b = C[b, a], b
        dest[a] = best_b
    root = np.arange(k)
    for a in range(k):
        r = a
        while dest[r] >= 0:
            r = dest[r]
        root[a] = r
    is_root = dest < 0
    n_vacated = int((~is_root).sum())
    order = np.lexsort((pruned, -s_raw[pruned]))
    salvaged = pruned[order[:n_vacated]]
    roots = kept[is_root]
    final_idx = np.sort(np.concatenate([roots, salvaged])).astype(np.int64)
    src_of = {int(i): [] for i in final_idx}
    for a in range(k):
        if not is_root[a]:
            src_of[int(kept[root[a]])].append(int(kept[a]))
    sources = [np.array(sorted(src_of[int(i)]), dtype=np.int64) for i in final_idx]
    return final_idx, sources


def sources_from_assign(assign: np.ndarray, pruned: np.ndarray, k: int) -> List[np.ndarray]:
    """Source sets I_src(c) for each kept slot c from an assignment vector."""
    return [pruned[assign == c] for c in range(k)]


# ---------------------------------------------------------------- Eq. 6
def weighted_merge(Xv: np.ndarray, s_hat: np.ndarray, final_idx: np.ndarray,
                   sources: Sequence[np.ndarray], mu: float = 1.0) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. 6 with a merge weight mu on the source terms (mu = 1 is the paper's form,
    mu = 0 disables merging).  Returns (y [k,D], wsum [k] the denominators)."""
    k = final_idx.size
    D = Xv.shape[1]
    y = np.zeros((k, D), dtype=np.float64)
    wsum = np.zeros(k, dtype=np.float64)
    for c in range(k):
        i = final_idx[c]
        num = s_hat[i] * Xv[i]
        den = s_hat[i]
        absorbed = 0.0
        for j in sources[c]:
            num = num + mu * s_hat[j] * Xv[j]
            den = den + mu * s_hat[j]
            absorbed = absorbed + mu * s_hat[j]
        wsum[c] = den
        # with no absorbed weight Eq. 6 is the identity h_i <- h_i (this also covers a
        # zero denominator); it is returned as such rather than as (s h) / s
        y[c] = num / den if absorbed > 0.0 else Xv[i]
    return y, wsum


# ---------------------------------------------------------------- output sequence
def assemble_sequence(X: np.ndarray, y: np.ndarray, final_idx: np.ndarray, P: int, V: int,
                      Tmax: int, text_len: int):
    """Output sequence [prefix | merged kept tokens in original order | valid text].

    X [N,D] full hidden states.  Returns (Y [P+k+Tmax, D] with rows past new_len zero,
    pos_out [P+k+Tmax] original position ids (-1 past new_len), new_len)."""
    k = final_idx.size
    new_len = P + k + text_len
    Y = np.zeros((P + k + Tmax, X.shape[1]), dtype=np.float64)
    pos = np.full(P + k + Tmax, -1, dtype=np.int64)
    Y[:P] = X[:P]
    pos[:P] = np.arange(P)
    Y[P:P + k] = y
    pos[P:P + k] = P + final_idx
    Y[P + k:new_len] = X[P + V:P + V + text_len]
    pos[P + k:new_len] = P + V + np.arange(text_len)
    return Y, pos, new_len


def gather_kv(cache: np.ndarray, pos_out: np.ndarray, new_len: int) -> np.ndarray:
    """cache [Hkv,N,d] -> rows at pos_out[0:new_len], in that order: [Hkv,new_len,d]."""
    return cache[:, pos_out[:new_len], :]


def gather_kv_paged(src_pool: np.ndarray, src_pages: np.ndarray, dst_pool: np.ndarray, dst_pages: np.ndarray,
                    pos_out: np.ndarray, new_len: int) -> None:
    """The same gather for one sequence of a paged cache (the block-table layout serving engines
    use; "KV-cache compatibility" of the stage).  Pools are [n_pages, Hkv, page_size, d]; token n of
    the sequence lives in page pages[n // page_size] at slot n % page_size.  Writes, in place,
    dst token n = src token pos_out[n] for n < new_len; nothing else of dst_pool changes."""
    ps = src_pool.shape[2]
    for n in range(new_len):
        m = int(pos_out[n])
        dst_pool[dst_pages[n // ps], :, n % ps, :] = src_pool[src_pages[m // ps], :, m % ps, :]


# ---------------------------------------------------------------- whole stage, one image
def stage(Q: np.ndarray, K: np.ndarray, X: np.ndarray, text_len: int, P: int, V: int, Tmax: int,
          k: int, lambda_max: float = 1.0, eps: float = EPS_DEFAULT, mask_on: bool = True,
          mu: float = 1.0, threshold: Optional[float] = None, route: str = "absorb",
          lse_extra: Optional[np.ndarray] = None, linear_mass: bool = False,
          score_rows: str = "all") -> dict:
    """All steps for one image.  Q [H,N,d], K [Hkv,N,d], X [N,D], N = P+V+Tmax.

    score_rows: which text rows rank the visual tokens (Sec. 4.1 does not say): "all" = the mean
    over every valid text row; "last" = the last valid text token's row alone, the criterion of the
    attention-score pruning the paper's ablation starts from (Sec. 5.3)."""
    Qv, Kv, Qt = Q[:, P:P + V], K[:, P:P + V], Q[:, P + V:]
    s = attention_mass_linear(Qv, Kv) if linear_mass else attention_mass(Qv, Kv)
    s_hat = salience(s, eps)
    bias = mask_log_discount(s_hat, lambda_max, eps, mask_on)
    if score_rows == "last":
        last = slice(text_len - 1, text_len)
        A = text_visual_attention(Qt[:, last], Kv, bias, 1, None if lse_extra is None else lse_extra[:, last])
    else:
        A = text_visual_attention(Qt, Kv, bias, text_len, lse_extra)
    r = selection_score(A)
    kept, pruned = select_topk(r, k)
    Xv = X[P:P + V]
    out = {"s_raw": s, "s_hat": s_hat, "score": r, "kept": kept, "pruned": pruned}
    if route == "absorb":
        t = -math.inf if threshold is None else threshold
        assign, best = route_absorb(Xv, kept, pruned, t)
        final_idx, sources = kept, sources_from_assign(assign, pruned, k)
        out.update(assign=assign, best=best)
    else:
        t = 0.8 if threshold is None else threshold
        final_idx, sources = route_paper(Xv, s, s_hat, kept, pruned, t)
    y, wsum = weighted_merge(Xv, s_hat, final_idx, sources, mu)
    Y, pos_out, new_len = assemble_sequence(X, y, final_idx, P, V, Tmax, text_len)
    out.update(final_idx=final_idx, sources=sources, y=y, wsum=wsum, Y=Y, pos_out=pos_out,
               new_len=new_len)
    return out


# ---------------------------------------------------------------- brute force, pins only
def full_bidirectional_attention(Q: np.ndarray, K: np.ndarray, P: int, V: int,
                                 lambda_max: float = 1.0, eps: float = EPS_DEFAULT,
                                 mask: str = "bidir") -> Tuple[np.ndarray, np.ndarray]:
    """Literal Eq. 1 / Eq. 4-5 on the whole sequence, one softmax row per query.

    Q [H,N,d], K [Hkv,N,d].  mask = "causal" gives Eq. 1; "bidir" replaces the -inf
    entries above the diagonal INSIDE the image span [P, P+V) by ln(max(lambda_j, eps)).
    Returns (A [H,N,N], s_hat [V])."""
    H, N, d = Q.shape
    Hkv = K.shape[0]
    s = attention_mass(Q[:, P:P + V], K[:, P:P + V])
    s_hat = salience(s, eps)
    M = np.zeros((N, N), dtype=np.float64)
    for i in range(N):
        for j in range(N):
            if i >= j:
                M[i, j] = 0.0
            elif mask == "bidir" and P <= i < P + V and P <= j < P + V:
                M[i, j] = math.log(max(lambda_max * s_hat[j - P], eps))
            else:
                M[i, j] = -math.inf
    A = np.zeros((H, N, N), dtype=np.float64)
    for h in range(H):
        W = (Q[h] @ K[kv_head(h, H, Hkv)].T) / math.sqrt(d)
        Z = W + M
        for i in range(N):
            z = Z[i]
            e = np.exp(z - z.max())
            A[h, i] = e / e.sum()
    return A, s_hat


def attention_forward(Q: np.ndarray, K: np.ndarray, Vval: np.ndarray, P: int, V: int,
                      lambda_max: float = 1.0, eps: float = EPS_DEFAULT,
                      mask: str = "bidir") -> Tuple[np.ndarray, np.ndarray]:
    """Output of one attention layer under the mask of Eq. 4-5 (or Eq. 1 for mask="causal"):
    out[h,i,:] = sum_j A[h,i,j] Vval[g(h),j,:] with A from full_bidirectional_attention.

    Q [H,N,d], K, Vval [Hkv,N,d].  Returns (out [H,N,d], s_hat [V])."""
    A, s_hat = full_bidirectional_attention(Q, K, P, V, lambda_max, eps, mask)
    H = Q.shape[0]
    Hkv = K.shape[0]
    out = np.stack([A[h] @ Vval[kv_head(h, H, Hkv)] for h in range(H)])
    return out, s_hat


# ---------------------------------------------------------------- Eq. 7 / Eq. 8
def layer_flops(v: int, d: int, m: int) -> float:
    """Per-layer theoretical FLOPs of the image tokens: 4 v d^2 + 2 v^2 d + 3 v d m."""
    return 4.0 * v * d * d + 2.0 * v * v * d + 3.0 * v * d * m


def theoretical_flops(layers: Sequence[int], tokens: Sequence[int], d: int, m: int) -> float:
    """Eq. 7: sum over stages n of L_n * layer_flops(v_n)."""
    return float(sum(L * layer_flops(v, d, m) for L, v in zip(layers, tokens)))


def flops_ratio(layers: Sequence[int], tokens: Sequence[int], v0: int, d: int, m: int) -> float:
    """Eq. 8: Eq. 7 over the unpruned cost of all layers at v0 tokens."""
    return theoretical_flops(layers, tokens, d, m) / (sum(layers) * layer_flops(v0, d, m))


# ---------------------------------------------------------------- Sec. 3.1: the RoPE score, and Eq. 2 from hidden states
def rope_rotate(v: np.ndarray, pos, theta: float = 10000.0) -> np.ndarray:
    """R_{Theta,m} v of Sec. 3.1 for vectors v [..., n, d] at positions pos [n]: the rotation by angle
    pos * theta^(-2c/d) of every coordinate pair; pairs are (c, c + d/2), the rotate-half layout of the
    LLaMA-family backbones the paper prunes (the paper writes R_{Theta,m-n} and leaves the pairing to them)."""
    d = v.shape[-1]
    half = d // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / d)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv_freq[None, :]            # [n, half]
    c, s = np.cos(ang), np.sin(ang)
    v1, v2 = v[..., :half], v[..., half:]
    return np.concatenate([v1 * c - v2 * s, v2 * c + v1 * s], axis=-1)


def project_queries(X: np.ndarray, Wq: np.ndarray, pos, H: int, d: int, theta: float = 10000.0) -> np.ndarray:
    """q_m = R_{Theta,m} W_q x_m (Sec. 3.1).  X [n, D] hidden states, Wq [H*d, D], pos [n] -> Q [H, n, d]."""
    U = (X @ Wq.T).reshape(X.shape[0], H, d).transpose(1, 0, 2)                      # [H, n, d]
    return rope_rotate(U, pos, theta)


def summed_visual_queries(Xv: np.ndarray, Wq: np.ndarray, pos, H: int, Hkv: int, d: int,
                          theta: float = 10000.0) -> np.ndarray:
    """sum over the visual tokens of their queries, per key/value head: the only thing Eq. 2 needs of
    the visual queries (sum_i W_ij = (sum_i q_i) . k_j / sqrt(d)).  Xv [V, D] -> [Hkv, d]."""
    Q = project_queries(Xv, Wq, pos, H, d, theta)                                    # [H, V, d]
    out = np.zeros((Hkv, d), dtype=np.float64)
    for h in range(H):
        out[kv_head(h, H, Hkv)] += Q[h].sum(axis=0)
    return out


def attention_mass_from_summed_queries(qbar: np.ndarray, Kv: np.ndarray, H: int) -> np.ndarray:
    """Eq. 2 from the summed visual queries qbar [Hkv, d] and the visual keys Kv [Hkv, V, d]."""
    d = Kv.shape[2]
    s = np.zeros(Kv.shape[1], dtype=np.float64)
    for g in range(Kv.shape[0]):
        s += (Kv[g] @ qbar[g]) / math.sqrt(d)
    return s / H
