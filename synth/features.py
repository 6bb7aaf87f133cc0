"""Synthetic stand-ins for gathered CLIP image/text features.

The paper trains on web image-text pairs with a ViT-B/32 image tower and a
text Transformer (Sec. 5.1) and reports batch sizes of 32,768 on 8 GPUs and
196,608 on 64 GPUs (Sec. 1, Table 3).  Neither the data nor the weights are
available here, so every input is drawn from a seeded generator that keeps the
shapes (B x d, d = 512 / 768), the unit row norm and the structure that matters
for the loss: each positive pair is strongly correlated, negatives are near
orthogonal, and optionally a fraction of rows are near duplicates of other
rows ("hard negatives").

Recipe (all float64 draws from numpy's PCG64 ``default_rng(seed)``):
  g_i ~ N(0,1)^d                               raw image direction
  hard rows (optional): a random subset of ``hard_frac * B`` indices j copies a
      source k drawn from the remaining indices: g_j = g_k + hard_sigma * n'_j
  I_i = g_i / |g_i|
  T_i = (g_i + noise * n_i) / |g_i + noise * n_i|,   n_i ~ N(0,1)^d
With noise = 0.5 the positive cosine is about 1/sqrt(1.25) = 0.894 and the
negative cosines are about N(0, 1/d).

bf16 workloads: rows are normalised in float32 and rounded to bfloat16 with
round-to-nearest-even; the 16-bit patterns are what the GPU library reads and
the exactly representable float32 upcasts are what a checker reads, so input
quantisation never counts as an error of the method.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Tuple

import numpy as np


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest even); returns the uint16 patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact float32 value of each bfloat16 pattern."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32)


def _normalise_rows(a: np.ndarray) -> np.ndarray:
    return a / np.linalg.norm(a, axis=1, keepdims=True)


def clip_pairs(B: int, d: int, seed: int, *, noise: float = 0.5,
               hard_frac: float = 0.0, hard_sigma: float = 0.329,
               chunk: int = 16384) -> Tuple[np.ndarray, np.ndarray]:
    """Draw B correlated (image, text) unit-norm feature pairs as float32.

    Drawn in row chunks so the float64 temporaries stay small at B = 196,608.
    Hard negatives need the raw directions of their sources, so when
    ``hard_frac > 0`` the raw matrix is kept in float32 during generation.
    """
    if B <= 0 or d <= 0:
        raise ValueError("B and d must be positive")
    rng = np.random.default_rng(seed)
    I = np.empty((B, d), dtype=np.float32)
    T = np.empty((B, d), dtype=np.float32)
    n_hard = int(round(hard_frac * B))
    if n_hard > 0:
        raw = np.empty((B, d), dtype=np.float32)
        for lo in range(0, B, chunk):
            hi = min(B, lo + chunk)
            raw[lo:hi] = rng.standard_normal((hi - lo, d))
        perm = rng.permutation(B)
        hard_idx, pool = perm[:n_hard], perm[n_hard:]
        src = pool[rng.integers(0, pool.size, size=n_hard)]
        for lo in range(0, n_hard, chunk):
            hi = min(n_hard, lo + chunk)
            raw[hard_idx[lo:hi]] = (raw[src[lo:hi]].astype(np.float64)
                                    + hard_sigma * rng.standard_normal((hi - lo, d)))
    else:
        raw = None
    for lo in range(0, B, chunk):
        hi = min(B, lo + chunk)
        g = (raw[lo:hi].astype(np.float64) if raw is not None
             else rng.standard_normal((hi - lo, d)))
        t = g + noise * rng.standard_normal((hi - lo, d))
        I[lo:hi] = _normalise_rows(g)
        T[lo:hi] = _normalise_rows(t)
    # float32 rounding moved the norms by ~1e-8; re-normalise in float32 so the
    # stored rows are unit-norm in the dtype that is handed over.
    I = _normalise_rows(I).astype(np.float32)
    T = _normalise_rows(T).astype(np.float32)
    return I, T


def two_views(M: int, d: int, seed: int, *, noise: float = 0.5) -> np.ndarray:
    """Features of two views of M samples for a self-supervised contrastive loss, as float32 (2M x d): view one
    (rows 0..M-1) and view two (rows M..2M-1) of sample i are the two members of clip_pairs' i-th pair, i.e.
    unit-norm rows with cosine about 0.894 between the views of a sample and near-orthogonal samples."""
    a, b = clip_pairs(M, d, seed, noise=noise)
    return np.ascontiguousarray(np.concatenate([a, b], axis=0), dtype=np.float32)


ADVERSARIAL_KINDS = ("norms", "permuted", "anti", "duplicates", "zero_rows", "big_norm_low_cos")


def adversarial_pairs(B: int, d: int, seed: int, kind: str, block: int = 256) -> Tuple[np.ndarray, np.ndarray]:
    """Feature pairs that are NOT CLIP-like, as float32: inputs a loss implementation must still get right.

    All start from clip_pairs(B, d, seed) (positive cosine about 0.894) and then
      norms            rows of I and T scaled by independent factors drawn uniformly from [0.3, 3]
      permuted         the text rows of every other block of `block` pairs rotated by one inside the block:
                       the positive pair of those rows is a random pair, its true partner (cosine 0.894)
                       sits next to it as a negative
      anti             every third text row negated: positives with cosine about -0.894
      duplicates       every 16th pair overwritten by a copy of the pair 5 places before it (both matrices):
                       exact duplicate keys, and negatives that tie with the positive
      zero_rows        one image row and a different text row set to zero
      big_norm_low_cos weak positives (noise 3.5: cosine about 0.27), every row scaled to norm 4
    """
    if kind not in ADVERSARIAL_KINDS:
        raise ValueError(f"unknown kind {kind}")
    rng = np.random.default_rng(seed + 1000)
    I, T = clip_pairs(B, d, seed, noise=3.5 if kind == "big_norm_low_cos" else 0.5)
    if kind == "norms":
        I = I * rng.uniform(0.3, 3.0, size=(B, 1)).astype(np.float32)
        T = T * rng.uniform(0.3, 3.0, size=(B, 1)).astype(np.float32)
    elif kind == "permuted":
        for lo in range(0, B, 2 * block):
            hi = min(B, lo + block)
            T[lo:hi] = np.roll(T[lo:hi], 1, axis=0)
    elif kind == "anti":
        T[::3] = -T[::3]
    elif kind == "duplicates":
        idx = np.arange(5, B, 16)
        I[idx] = I[idx - 5]
        T[idx] = T[idx - 5]
    elif kind == "zero_rows":
        I[B // 3] = 0.0
        T[(2 * B) // 3 + 1] = 0.0
    elif kind == "big_norm_low_cos":
        I, T = 4.0 * I, 4.0 * T
    return np.ascontiguousarray(I, dtype=np.float32), np.ascontiguousarray(T, dtype=np.float32)


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    B: int
    d: int
    N: int
    dtype: str          # "f32" or "bf16"
    s: float
    seed: int
    noise: float = 0.5
    hard_frac: float = 0.0

    @property
    def b(self) -> int:
        return self.B // self.N


CONFIGS: Dict[str, WorkloadConfig] = {
    # small case: fp32, every rank, a float64 checker finishes in well under a second
    "tiny": WorkloadConfig("tiny", 256, 512, 4, "f32", 1.0 / 0.07, 0),
    # ViT-B/32 batch share of the 8-GPU run: one rank's 4096 x 32768 blocks
    "b32k_n8": WorkloadConfig("b32k_n8", 32768, 512, 8, "bf16", 1.0 / 0.07, 1),
    # the same batch without decomposition (every row on one device)
    "full_n1": WorkloadConfig("full_n1", 32768, 512, 1, "bf16", 1.0 / 0.07, 1),
    # the 64-GPU, 196,608 batch: one rank's 3072 x 196608 blocks, scale at the clamp
    "b196k_n64": WorkloadConfig("b196k_n64", 196608, 512, 64, "bf16", 100.0, 2),
    # same shape with weak positives so that s = 100 does not saturate the softmax
    "b196k_n64_hard": WorkloadConfig("b196k_n64_hard", 196608, 512, 64, "bf16", 100.0, 2, noise=3.5),
    # wider embedding with 10% near-duplicate rows
    "b64k_d768_n8": WorkloadConfig("b64k_d768_n8", 65536, 768, 8, "bf16", 1.0 / 0.07, 3, hard_frac=0.10),
    # the shape of the paper's own timing table (Table 4: 64 GPUs, batch 32,768, 512 pairs per GPU)
    "b32k_n64": WorkloadConfig("b32k_n64", 32768, 512, 64, "bf16", 1.0 / 0.07, 1),
    # a batch whose rank share is not a whole number of 256-row tiles (3750 pairs per rank)
    "b30k_n8_ragged": WorkloadConfig("b30k_n8_ragged", 30000, 512, 8, "bf16", 1.0 / 0.07, 5),
    # the batch of the paper's accuracy tables (Tables 5-7: 65,536 on 64 GPUs)
    "b64k_n64": WorkloadConfig("b64k_n64", 65536, 512, 64, "bf16", 1.0 / 0.07, 4),
}


def make_config_inputs(cfg: WorkloadConfig):
    """Returns (I_f32, T_f32, I_bits, T_bits).

    For "bf16" workloads the float32 arrays are the exact upcasts of the 16-bit
    patterns; for "f32" workloads the bit arrays are None.
    """
    I, T = clip_pairs(cfg.B, cfg.d, cfg.seed, noise=cfg.noise, hard_frac=cfg.hard_frac)
    if cfg.dtype == "bf16":
        Ib, Tb = f32_to_bf16_bits(I), f32_to_bf16_bits(T)
        return bf16_bits_to_f32(Ib), bf16_bits_to_f32(Tb), Ib, Tb
    if cfg.dtype != "f32":
        raise ValueError(f"unknown dtype {cfg.dtype}")
    return I, T, None, None
