"""TEST INFRASTRUCTURE -- CPU oracle of what surrounds the draft head inside one draft step
(not part of the product).

Section 2.3 of the paper lists the draft model's components: (1) a feature-fusion layer, a linear
projection from three concatenated target features to the hidden size (3d -> d, Table 1's
"Feature fusion" row: 2*3d*d = 100.7 M FLOPs at d = 4096), (2) one decoder layer, (3) the LM head.
The hidden state that reaches the head has passed the model's final normalisation, and drafting
a tree scores each proposed token by the log-probability of its whole path.  The head's
neighbours on both sides, in plain numpy / the C oracle:

  feature_fusion  g[r,j] = sum_i x[r,i] * W_fc[j,i]   bf16 inputs, sequential fp32 accumulation,
                  one rounding to bf16 (the next layer's input format)
  rmsnorm         h[r,i] = bf16( g[r,i] * rsqrt(mean_i g[r,i]^2 + eps) * gamma[i] ), mean in double,
                  the rest in fp32 with one rounding to bf16 at the end (the paper does not say how the
                  draft normalises; this is the root-mean-square norm of the LLaMA family it drafts for)
  head_fused      the draft step over the normalised hidden state, with each proposed token's
                  log-probability added to the cumulative log-probability of the node it extends
                  (score of a child = score of its parent + log p(child | parent))

Only tests, the smoke check and the benchmark's CPU-baseline leg import this module; it imports
nothing from the product.  Pinned by tests/test_prologue_pins.py.
"""
from __future__ import annotations

import numpy as np

from oracle import vt_oracle as vo


def _bf16_to_f32(u16: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(u16, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _f32_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round to nearest even (finite inputs)."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rnd = ((b >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((b + rnd) >> np.uint32(16)).astype(np.uint16)


def fusion_flops(d_in: int, d_out: int) -> int:
    """Multiplies plus adds of the projection per row (Section 2.3: 2 * 3d * d for d_in = 3d)."""
    return 2 * d_in * d_out


def feature_fusion(x_u16: np.ndarray, Wfc_u16: np.ndarray) -> np.ndarray:
    """x[R,d_in], W_fc[d_out,d_in] (bf16 bits) -> g[R,d_out] (bf16 bits)."""
    return _f32_to_bf16(vo.logits(x_u16, Wfc_u16))


def rmsnorm(g_u16: np.ndarray, gamma_u16: np.ndarray, eps: float) -> np.ndarray:
    """g[R,H], gamma[H] (bf16 bits) -> h[R,H] (bf16 bits)."""
    g = _bf16_to_f32(g_u16)
    gam = _bf16_to_f32(gamma_u16)
    ms = np.mean(g.astype(np.float64) ** 2, axis=1)
    r = (1.0 / np.sqrt(ms + float(eps))).astype(np.float32)
    return _f32_to_bf16((g * r[:, None]).astype(np.float32) * gam[None, :])


def head_fused(g_u16: np.ndarray, gamma_u16: np.ndarray, eps: float, W_sub: np.ndarray, d2t: np.ndarray, k: int,
               parent_scores: np.ndarray | None = None):
    """Normalise, run the draft head, add the parents' cumulative log-probabilities.
    Returns the head's result with .scores[R,k] (fp32) = parent + logp, and .h (the normalised state)."""
    h = rmsnorm(g_u16, gamma_u16, eps)
    res = vo.draft_head(h, W_sub, d2t, k)
    parent = np.zeros(h.shape[0], dtype=np.float32) if parent_scores is None else np.asarray(parent_scores, dtype=np.float32)
    scores = (res.logp + parent[:, None]).astype(np.float32)
    return res, scores, h
