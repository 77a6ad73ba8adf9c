"""Seeded synthetic inputs shaped like the paper's workloads.

This module only *makes inputs*: hidden states drawn from a cluster mixture, the
query/key projections with rotary position embedding (the RoPE score of
Sec. 3.1), random K/V caches, ragged text lengths and dtype quantisation.  It
holds none of the pruning method's arithmetic (no salience, mask, softmax,
top-k, similarity or merge) and imports neither the oracle nor the HIP binding;
both are fed from here so that they see bit-identical inputs.

The images, prompts and weights of the paper's evaluation (LLaVA-1.5 at 576
visual tokens, LLaVA-NeXT at ~2304, Sec. 5.1) are not available, so these
inputs stand in for them: same shapes, token counts and budgets; redundancy is
modelled by a Gaussian cluster mixture and high-norm tokens by 8x outliers.
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass
from typing import Dict, List, Optional

import numpy as np

F32 = "f32"
BF16 = "bf16"


@dataclass(frozen=True)
class StageConfig:
    """Shape and recipe of one pruning-stage workload (one batch)."""
    name: str
    B: int            # images per batch
    D: int            # hidden size
    H: int            # query heads
    Hkv: int          # key/value heads
    d: int            # head dim
    P: int            # prefix (system prompt) tokens before the image
    V: int            # visual tokens
    Tmax: int         # padded text length
    k: int            # visual tokens kept
    qk_dtype: str
    h_dtype: str
    kv_dtype: str
    n_clusters: int
    outliers: bool    # every 64th visual token scaled 8x
    L_kv: int         # layers of K/V cache in front of the pruning layer
    seed: int
    ragged_text: bool = False
    text_lo: int = 16
    rope_theta: float = 10000.0

    @property
    def N(self) -> int:
        return self.P + self.V + self.Tmax

    @property
    def N_out(self) -> int:
        return self.P + self.k + self.Tmax


# Workloads.  C1..C5 follow the benchmark's five configurations, C6 is the
# 2304-token batch-16 target; the S* ones are small cases for element-wise parity.
CONFIGS: Dict[str, StageConfig] = {c.name: c for c in [
    StageConfig("C1", 1, 4096, 32, 32, 128, 35, 576, 32, 144, F32, F32, F32, 48, False, 2, 0),
    StageConfig("C2", 1, 4096, 32, 32, 128, 35, 2304, 64, 320, BF16, BF16, BF16, 192, True, 2, 1),
    StageConfig("C3", 16, 4096, 32, 32, 128, 35, 576, 128, 144, F32, F32, BF16, 48, False, 2, 2,
                ragged_text=True, text_lo=16),
    StageConfig("C4", 4, 3584, 28, 4, 128, 0, 4096, 48, 512, BF16, BF16, BF16, 256, False, 2, 3),
    StageConfig("C5a", 8, 5120, 40, 40, 128, 0, 2304, 64, 576, BF16, BF16, BF16, 192, True, 2, 4),
    StageConfig("C5b", 8, 5120, 40, 40, 128, 0, 576, 64, 160, BF16, BF16, BF16, 192, True, 16, 4),
    StageConfig("C6", 16, 4096, 32, 32, 128, 35, 2304, 64, 320, BF16, BF16, BF16, 192, True, 2, 5),
    # small parity cases: several tiles and ragged tails in every dimension
    StageConfig("S0", 2, 256, 4, 4, 64, 3, 72, 8, 20, F32, F32, F32, 6, False, 1, 100),
    StageConfig("S1", 3, 512, 8, 8, 128, 5, 333, 24, 77, F32, F32, BF16, 12, True, 2, 101,
                ragged_text=True, text_lo=3),
    StageConfig("S2", 2, 768, 8, 2, 128, 7, 461, 40, 129, BF16, BF16, BF16, 16, True, 2, 102,
                ragged_text=True, text_lo=5),
    StageConfig("S3", 2, 384, 6, 3, 64, 0, 200, 1, 199, BF16, BF16, F32, 5, False, 1, 103),
    StageConfig("S4", 1, 1024, 16, 16, 128, 35, 576, 32, 144, BF16, BF16, BF16, 48, False, 2, 104),
]}


# --------------------------------------------------------------------------
# dtype plumbing (bf16 is carried on the host as uint16 bit patterns)
# --------------------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns uint16 bits."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounding = ((u >> 16) & 1) + np.uint32(0x7FFF)
    out = ((u + rounding) >> 16).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out[nan] = 0x7FC0
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


def quantise(x: np.ndarray, dtype: str) -> np.ndarray:
    """Cast to the storage dtype: float32 array, or uint16 bf16 bit patterns."""
    if dtype == F32:
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == BF16:
        return f32_to_bf16_bits(np.asarray(x, dtype=np.float32))
    raise ValueError(dtype)


def to_f64(x: np.ndarray, dtype: str) -> np.ndarray:
    """Exact upcast of a stored array (see quantise) to float64."""
    if dtype == F32:
        return x.astype(np.float64)
    if dtype == BF16:
        return bf16_bits_to_f32(x).astype(np.float64)
    raise ValueError(dtype)


def itemsize(dtype: str) -> int:
    return 4 if dtype == F32 else 2


# --------------------------------------------------------------------------
# rotary position embedding (input synthesis; Sec. 3.1)
# --------------------------------------------------------------------------

def rope_rotate(x: np.ndarray, positions: np.ndarray, theta: float) -> np.ndarray:
    """Rotate-half RoPE.  x: [..., n, d]; positions: [n]; pairs (i, i + d/2),
    angular frequency theta**(-2i/d)."""
    d = x.shape[-1]
    half = d // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / d)
    ang = positions.astype(np.float64)[:, None] * inv_freq[None, :]     # [n, half]
    c = np.cos(ang).astype(x.dtype)
    s = np.sin(ang).astype(x.dtype)
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def project_qk(X: np.ndarray, positions: np.ndarray, Wq: np.ndarray, Wk: np.ndarray,
               H: int, Hkv: int, d: int, theta: float):
    """X: [n, D] float32 -> Q [H, n, d], K [Hkv, n, d] (float32) with RoPE applied
    at the given position ids."""
    n = X.shape[0]
    q = (X @ Wq).reshape(n, H, d).transpose(1, 0, 2)
    k = (X @ Wk).reshape(n, Hkv, d).transpose(1, 0, 2)
    return rope_rotate(q, positions, theta), rope_rotate(k, positions, theta)


# --------------------------------------------------------------------------
# the generator
# --------------------------------------------------------------------------

def make_weights(cfg: StageConfig, rng: np.random.Generator):
    Wq = (rng.standard_normal((cfg.D, cfg.H * cfg.d), dtype=np.float32) / np.sqrt(cfg.D)).astype(np.float32)
    Wk = (rng.standard_normal((cfg.D, cfg.Hkv * cfg.d), dtype=np.float32) / np.sqrt(cfg.D)).astype(np.float32)
    return Wq, Wk


def make_hidden(cfg: StageConfig, rng: np.random.Generator) -> np.ndarray:
    """One image's hidden states [N, D] float32: prefix | visual mixture | text."""
    X = np.empty((cfg.N, cfg.D), dtype=np.float32)
    X[:cfg.P] = rng.standard_normal((cfg.P, cfg.D), dtype=np.float32)
    centres = rng.standard_normal((cfg.n_clusters, cfg.D), dtype=np.float32)
    which = rng.integers(0, cfg.n_clusters, size=cfg.V)
    vis = centres[which] + np.float32(0.3) * rng.standard_normal((cfg.V, cfg.D), dtype=np.float32)
    if cfg.outliers:
        vis[::64] *= np.float32(8.0)
    X[cfg.P:cfg.P + cfg.V] = vis
    X[cfg.P + cfg.V:] = rng.standard_normal((cfg.Tmax, cfg.D), dtype=np.float32)
    return X


def make_inputs(cfg: StageConfig, with_kv: bool = True) -> dict:
    """Build one batch.  Returns stored arrays (see quantise) and metadata:

    q      [B, H,   N, d]  qk_dtype    k  [B, Hkv, N, d]  qk_dtype
    hidden [B, N, D]       h_dtype     text_len [B] int32 (valid text tokens)
    k_cache, v_cache: lists of L_kv arrays [B, Hkv, N, d] kv_dtype
    Rows of padded text positions hold ordinary random values that a correct
    implementation never lets into a result.
    """
    ss = np.random.SeedSequence(cfg.seed)
    children = ss.spawn(cfg.B + 2)
    Wq, Wk = make_weights(cfg, np.random.default_rng(children[0]))
    rng_meta = np.random.default_rng(children[1])
    if cfg.ragged_text:
        text_len = rng_meta.integers(cfg.text_lo, cfg.Tmax + 1, size=cfg.B).astype(np.int32)
        text_len[0] = cfg.Tmax            # always exercise the full-length row block
        if cfg.B > 1:
            text_len[1] = cfg.text_lo     # and the shortest
    else:
        text_len = np.full(cfg.B, cfg.Tmax, dtype=np.int32)
    positions = np.arange(cfg.N)
    q = np.empty((cfg.B, cfg.H, cfg.N, cfg.d), dtype=np.float32)
    k = np.empty((cfg.B, cfg.Hkv, cfg.N, cfg.d), dtype=np.float32)
    hidden = np.empty((cfg.B, cfg.N, cfg.D), dtype=np.float32)
    for b in range(cfg.B):
        rng = np.random.default_rng(children[2 + b])
        X = make_hidden(cfg, rng)
        hidden[b] = X
        q[b], k[b] = project_qk(X, positions, Wq, Wk, cfg.H, cfg.Hkv, cfg.d, cfg.rope_theta)
    out = {
        "cfg": cfg,
        "q": quantise(q, cfg.qk_dtype),
        "k": quantise(k, cfg.qk_dtype),
        "hidden": quantise(hidden, cfg.h_dtype),
        "text_len": text_len,
        "Wq": Wq, "Wk": Wk,
    }
    del q, k, hidden
    if with_kv:
        out["k_cache"], out["v_cache"] = make_kv_cache(cfg, cfg.N, children[1])
    return out


def make_kv_cache(cfg: StageConfig, n_rows: int, seed_seq) -> tuple:
    """Random K/V caches of the layers in front of the pruning layer; every row
    is distinct so a misplaced row shows."""
    rng = np.random.default_rng(np.random.SeedSequence(entropy=seed_seq.entropy,
                                                       spawn_key=tuple(seed_seq.spawn_key) + (7,)))
    kc: List[np.ndarray] = []
    vc: List[np.ndarray] = []
    shape = (cfg.B, cfg.Hkv, n_rows, cfg.d)
    for _ in range(cfg.L_kv):
        kc.append(quantise(rng.standard_normal(shape, dtype=np.float32), cfg.kv_dtype))
        vc.append(quantise(rng.standard_normal(shape, dtype=np.float32), cfg.kv_dtype))
    return kc, vc


def second_stage_inputs(cfg2: StageConfig, hidden_out: np.ndarray, pos_out: np.ndarray,
                        new_len: np.ndarray, text_len: np.ndarray) -> dict:
    """Inputs of a second pruning stage from the first stage's output sequence.

    hidden_out [B, N2, D] stored in cfg2.h_dtype, pos_out [B, N2] original
    position ids, N2 = cfg2.N.  Fresh projection weights (a deeper layer) are
    drawn from cfg2.seed; Q/K are rotated at the ORIGINAL position ids.
    """
    ss = np.random.SeedSequence(cfg2.seed + 1000)
    children = ss.spawn(2)
    Wq, Wk = make_weights(cfg2, np.random.default_rng(children[0]))
    B = cfg2.B
    q = np.empty((B, cfg2.H, cfg2.N, cfg2.d), dtype=np.float32)
    k = np.empty((B, cfg2.Hkv, cfg2.N, cfg2.d), dtype=np.float32)
    Xf = to_f64(hidden_out, cfg2.h_dtype).astype(np.float32)
    for b in range(B):
        pos = pos_out[b].astype(np.int64).copy()
        n_valid = int(new_len[b])
        # padded rows: continue the position sequence so the values stay finite
        pos[n_valid:] = pos[n_valid - 1] + 1 + np.arange(cfg2.N - n_valid)
        q[b], k[b] = project_qk(Xf[b], pos, Wq, Wk, cfg2.H, cfg2.Hkv, cfg2.d, cfg2.rope_theta)
    out = {
        "cfg": cfg2,
        "q": quantise(q, cfg2.qk_dtype),
        "k": quantise(k, cfg2.qk_dtype),
        "hidden": hidden_out,
        "text_len": text_len.astype(np.int32),
        "Wq": Wq, "Wk": Wk,
    }
    out["k_cache"], out["v_cache"] = make_kv_cache(cfg2, cfg2.N, children[1])
    return out


def shrink(cfg: StageConfig, **kw) -> StageConfig:
    return dataclasses.replace(cfg, **kw)
