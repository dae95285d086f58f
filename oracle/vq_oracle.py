"""TEST INFRASTRUCTURE -- CPU oracle of the compressed draft head (not part of the product).

The paper's point (Sections 1, 2.3) is that the draft's LM head dominates its latency and that
its cost is 2*d*k per token; at one row that cost is the bytes of W_sub.  Trimming cuts k; storing
W_sub in a narrower format cuts the bytes per weight.  This file states, in plain numpy, what the
two compressed forms are and what the head over them computes:

  FP8   every weight as an OCP 8-bit float E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa
        bits; subnormals at exponent 0; no infinities; largest finite value 448; codes 0x7f / 0xff
        are NaN and never produced), with one fp32 scale per row of W_sub:
            scale_j = max_i |W[j,i]| / 448   (1 if the row is all zero)
            code    = E4M3(W[j,i] / scale_j)  round to nearest, ties to even, saturating
  MXFP4 OCP microscaling: blocks of 32 consecutive weights of a row share a power-of-two scale
        stored as an 8-bit biased exponent (E8M0, bias 127), the weights are 4-bit floats E2M1
        (1 sign, 2 exponent bits with bias 1, 1 mantissa bit: 0, 0.5, 1, 1.5, 2, 3, 4, 6):
            e_block = floor(log2(max |w| over the block)) - 2     (2 = exponent of 6, the largest E2M1)
            code    = E2M1(w / 2^e_block)  round to nearest, ties to even, saturating at 6
        two codes per byte, the even element in the low nibble; an all-zero block stores exponent
        byte 127.

The head over a compressed W_sub is the bf16 head's definition applied to the dequantised
weights (code value times scale, rounded once to fp32): logits by sequential fp32 accumulation,
log-softmax over V_d, k best by (logit, lower draft index), d2t remap -- oracle/vt_oracle.c.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this module; it imports
nothing from the product.  Pinned by tests/test_quant_pins.py (format tables, a library's own
E4M3 conversion, exhaustive nearest-value search in exact rational arithmetic, round trips, the
formats' error bounds, restriction / normalisation invariants of the head).
"""
from __future__ import annotations

import numpy as np

from oracle import vt_oracle as vo

FMT_FP8 = 1
FMT_MXFP4 = 2
E4M3_MAX = 448.0
MX_BLOCK = 32


def _bf16_to_f32(u16: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(u16, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ---------------------------------------------------------------- E4M3
def e4m3_value(code: int) -> float:
    """The real number an E4M3 code stands for (nan for the two NaN codes)."""
    s = -1.0 if code & 0x80 else 1.0
    e = (code >> 3) & 0xF
    m = code & 0x7
    if e == 0xF and m == 0x7:
        return float("nan")
    if e == 0:
        return s * (m / 8.0) * 2.0 ** (-6)
    return s * (1.0 + m / 8.0) * 2.0 ** (e - 7)


def e4m3_table() -> np.ndarray:
    return np.array([e4m3_value(c) for c in range(256)], dtype=np.float32)


def e4m3_encode(x: np.ndarray) -> np.ndarray:
    """Finite fp32 values -> E4M3 codes: nearest representable value, ties to the even mantissa,
    magnitudes beyond 448 saturate to 448."""
    x = np.asarray(x, dtype=np.float32)
    a = np.abs(x).astype(np.float64)  # exact; all steps below are exact in double
    sign = (np.signbit(x)).astype(np.uint8) << 7
    _, ex = np.frexp(a)                                  # a = f * 2**ex, f in [0.5, 1)
    e = np.maximum(ex - 1, -6)                           # binade; everything below 2**-6 shares the subnormal step
    step = np.ldexp(1.0, e - 3)                          # spacing of E4M3 values in that binade
    q = np.rint(a / step) * step                         # round half to even multiple of the spacing
    q = np.minimum(q, E4M3_MAX)
    # the code of the representable value q
    _, qx = np.frexp(q)
    qe = qx - 1
    normal = q >= 2.0 ** (-6)
    mant_n = np.rint((q / np.ldexp(1.0, qe) - 1.0) * 8.0).astype(np.int64)
    code_n = ((qe + 7) << 3) | mant_n
    code_s = np.rint(q * 2.0 ** 9).astype(np.int64)
    code = np.where(normal, code_n, code_s).astype(np.uint8)
    return (code | sign).astype(np.uint8)


def quantize_fp8(W_u16: np.ndarray):
    """bf16 rows -> (codes[V,H] uint8, scales[V] float32)."""
    w = _bf16_to_f32(W_u16)
    amax = np.max(np.abs(w), axis=1)
    scale = (amax / np.float32(E4M3_MAX)).astype(np.float32)
    scale = np.where(amax > 0, scale, np.float32(1.0)).astype(np.float32)
    x = (w / scale[:, None]).astype(np.float32)          # one fp32 division per weight
    return e4m3_encode(x), scale


def dequantize_fp8(codes: np.ndarray, scales: np.ndarray) -> np.ndarray:
    return (e4m3_table()[codes] * np.asarray(scales, dtype=np.float32)[:, None]).astype(np.float32)


# ---------------------------------------------------------------- MXFP4
E2M1_VALUES = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0], dtype=np.float64)


def e2m1_value(nibble: int) -> float:
    s = -1.0 if nibble & 0x8 else 1.0
    e = (nibble >> 1) & 0x3
    m = nibble & 0x1
    if e == 0:
        return s * 0.5 * m
    return s * (1.0 + 0.5 * m) * 2.0 ** (e - 1)


def e2m1_encode(x: np.ndarray) -> np.ndarray:
    """Finite values -> E2M1 nibbles: nearest of the eight magnitudes, ties to the even mantissa
    bit, magnitudes beyond 6 saturate to 6."""
    x = np.asarray(x, dtype=np.float64)
    a = np.abs(x)
    sign = np.signbit(x).astype(np.uint8) << 3
    _, ex = np.frexp(a)
    e = np.clip(ex - 1, 0, 2)                            # binades [0,2) (subnormal step), [2,4), [4,8)
    step = np.ldexp(0.5, e)                              # 0.5, 1, 2
    q = np.minimum(np.rint(a / step) * step, 6.0)
    code = np.searchsorted(E2M1_VALUES, q).astype(np.uint8)   # q is exactly one of the eight values
    return code | sign


def quantize_mxfp4(W_u16: np.ndarray):
    """bf16 rows (H a multiple of 32) -> (packed[V,H/2] uint8, block exponents[V,H/32] uint8)."""
    w = _bf16_to_f32(W_u16).astype(np.float64)
    V, H = w.shape
    assert H % MX_BLOCK == 0
    blocks = w.reshape(V, H // MX_BLOCK, MX_BLOCK)
    amax = np.max(np.abs(blocks), axis=2)
    _, ex = np.frexp(amax)                               # floor(log2 amax) = ex - 1 for amax > 0
    e_block = np.where(amax > 0, ex - 1 - 2, 0)
    e_byte = np.clip(e_block + 127, 0, 254).astype(np.uint8)
    x = blocks / np.ldexp(1.0, e_byte.astype(np.int64) - 127)[:, :, None]
    nib = e2m1_encode(x).reshape(V, H)
    packed = (nib[:, 0::2] | (nib[:, 1::2] << 4)).astype(np.uint8)
    return packed, e_byte


def dequantize_mxfp4(packed: np.ndarray, e_bytes: np.ndarray) -> np.ndarray:
    V, Hh = packed.shape
    H = Hh * 2
    nib = np.empty((V, H), dtype=np.uint8)
    nib[:, 0::2] = packed & 0xF
    nib[:, 1::2] = packed >> 4
    table = np.array([e2m1_value(n) for n in range(16)], dtype=np.float64)
    vals = table[nib].reshape(V, H // MX_BLOCK, MX_BLOCK)
    out = vals * np.ldexp(1.0, e_bytes.astype(np.int64) - 127)[:, :, None]
    return out.reshape(V, H).astype(np.float32)


# ---------------------------------------------------------------- subset construction and head
def quantize(W_u16: np.ndarray, fmt: int):
    if fmt == FMT_FP8:
        return quantize_fp8(W_u16)
    if fmt == FMT_MXFP4:
        return quantize_mxfp4(W_u16)
    raise ValueError("unknown format")


def dequantize(codes: np.ndarray, scales: np.ndarray, fmt: int) -> np.ndarray:
    if fmt == FMT_FP8:
        return dequantize_fp8(codes, scales)
    if fmt == FMT_MXFP4:
        return dequantize_mxfp4(codes, scales)
    raise ValueError("unknown format")


def build_subset_q(W_u16: np.ndarray, ids: np.ndarray, fmt: int):
    """Section 2.1's subset, stored compressed: the rows of V_d in the order of `ids`, quantised
    row by row; (codes, scales, d2t)."""
    W_sub, d2t = vo.build_subset(W_u16, ids)
    codes, scales = quantize(W_sub, fmt)
    return codes, scales, d2t


def draft_head_q(h_u16: np.ndarray, codes: np.ndarray, scales: np.ndarray, fmt: int, d2t: np.ndarray, k: int,
                 want_logits: bool = True):
    """The draft step over a compressed W_sub: the bf16 head's definition on the dequantised weights."""
    return vo.draft_head_w32(h_u16, dequantize(codes, scales, fmt), d2t, k, want_logits=want_logits)
