"""Seeded synthetic inputs for the trimmed-vocabulary draft LM head.

This module only *draws inputs*: the full unembedding matrix W[V,H], hidden
states h[R,H] and the list of surviving token ids (the draft vocabulary V_d of
Section 2.1).  It contains none of the head's arithmetic (no projection, no
softmax, no top-k, no gather) so that the CPU oracle's tests and the HIP path's
tests can both feed from it without sharing any of the method.

Everything is counter based: element e of stream s under seed S is a pure
function of (S, s, e), so any row range can be produced on its own and in
parallel.  The generator is SplitMix64 (Steele, Lea, Flood 2014: additive
constant 0x9E3779B97F4A7C15 and the two-multiply finaliser) feeding a
Box-Muller transform; bf16 values are made by one round-to-nearest-even of the
fp32 draw.

The paper's workloads (Section 3: a LLaMA-3 head with V = 128 256, d = 4096,
draft vocabularies of 4 380 .. 13 264 tokens chosen by corpus frequency) need a
tokenizer and corpora that are not available; the Zipf-ranked subset below
stands in for the frequency ranking of Section 2.2.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

# sub-stream numbers
STREAM_W = 0
STREAM_H = 1
STREAM_PERM = 2
STREAM_KEYS = 3
STREAM_PEAKED = 4
STREAM_TOKENS = 5

FULL_VOCAB = 128256  # LLaMA-3 vocabulary size (Section 2.3, Table 1)


def _finalise(z: np.ndarray) -> np.ndarray:
    """SplitMix64 output function on a uint64 array (wrap-around arithmetic)."""
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _stream_base(seed: int, stream: int) -> np.uint64:
    with np.errstate(over="ignore"):
        s = np.array([np.uint64(seed) * np.uint64(0xD1342543DE82EF95) + np.uint64(stream) + np.uint64(1)],
                     dtype=np.uint64)
        return _finalise(s * _GOLDEN)[0]


def raw_u64(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """count 64-bit words: word n is SplitMix64's (n+1)-th output from the stream's base state."""
    with np.errstate(over="ignore"):
        base = _stream_base(seed, stream)
        n = np.arange(start + 1, start + 1 + count, dtype=np.uint64)
        return _finalise(base + n * _GOLDEN)


def uniform01(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """Doubles in (0, 1]: (top 53 bits + 1) * 2**-53."""
    u = raw_u64(seed, stream, start, count) >> np.uint64(11)
    return (u.astype(np.float64) + 1.0) * (2.0 ** -53)


def normal(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """Standard normals (float64) for flat element indices [start, start+count).

    Elements 2i and 2i+1 are the cosine and sine branch of one Box-Muller pair
    built from uniform words 2i and 2i+1.
    """
    first = start - (start & 1)
    last = start + count
    last += last & 1
    npair = (last - first) // 2
    u = uniform01(seed, stream, first, 2 * npair)
    u1 = u[0::2]
    u2 = u[1::2]
    r = np.sqrt(-2.0 * np.log(u1))
    t = (2.0 * np.pi) * u2
    out = np.empty(2 * npair, dtype=np.float64)
    out[0::2] = r * np.cos(t)
    out[1::2] = r * np.sin(t)
    off = start - first
    return out[off:off + count]


def f32_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns (finite inputs)."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rnd = ((b >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((b + rnd) >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(u: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to fp32."""
    return (np.ascontiguousarray(u, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _n_threads() -> int:
    return max(1, min(16, os.cpu_count() or 1))


def _rows_bf16(seed: int, stream: int, row0: int, row1: int, H: int, scale: float) -> np.ndarray:
    x = normal(seed, stream, row0 * H, (row1 - row0) * H)
    return f32_to_bf16((x * scale).astype(np.float32)).reshape(row1 - row0, H)


def gen_W(seed: int, V: int, H: int, std: float = 0.02, row0: int = 0, row1: int | None = None) -> np.ndarray:
    """Rows [row0,row1) of the full unembedding matrix: i.i.d. N(0, std) -> bf16 (uint16 bits)."""
    row1 = V if row1 is None else row1
    n = row1 - row0
    out = np.empty((n, H), dtype=np.uint16)
    step = max(1, (1 << 21) // H)
    blocks = [(a, min(a + step, row1)) for a in range(row0, row1, step)]

    def work(b):
        out[b[0] - row0:b[1] - row0] = _rows_bf16(seed, STREAM_W, b[0], b[1], H, std)

    if len(blocks) > 1:
        with ThreadPoolExecutor(_n_threads()) as ex:
            list(ex.map(work, blocks))
    else:
        for b in blocks:
            work(b)
    return out


def gen_W_rows(seed: int, H: int, rows: np.ndarray, std: float = 0.02) -> np.ndarray:
    """The given rows of W (same bits as gen_W would give), without generating the rest."""
    rows = np.asarray(rows, dtype=np.int64)
    out = np.empty((len(rows), H), dtype=np.uint16)
    for n, r in enumerate(rows):
        out[n] = _rows_bf16(seed, STREAM_W, int(r), int(r) + 1, H, std)[0]
    return out


def gen_h(seed: int, R: int, H: int, peaked_frac: float = 0.0, peaked_scale: float = 10.0) -> np.ndarray:
    """Hidden states h[R,H]: i.i.d. N(0,1) -> bf16.  With peaked_frac > 0, floor(frac*R) rows
    (the first ones of a seeded permutation) are multiplied by peaked_scale in fp32 before the
    single rounding to bf16 (rows with sharply peaked logits)."""
    x = normal(seed, STREAM_H, 0, R * H).astype(np.float32).reshape(R, H)
    n_peak = int(np.floor(peaked_frac * R))
    if n_peak > 0:
        order = np.argsort(raw_u64(seed, STREAM_PEAKED, 0, R), kind="stable")
        x[order[:n_peak]] *= np.float32(peaked_scale)
    return f32_to_bf16(x).reshape(R, H)


def peaked_rows(seed: int, R: int, peaked_frac: float) -> np.ndarray:
    """Which rows gen_h scaled (sorted)."""
    n_peak = int(np.floor(peaked_frac * R))
    order = np.argsort(raw_u64(seed, STREAM_PEAKED, 0, R), kind="stable")
    return np.sort(order[:n_peak])


def zipf_subset(seed: int, V: int, V_draft: int, s: float = 1.1) -> np.ndarray:
    """V_draft distinct token ids in [0,V), int32, sorted ascending.

    A seeded permutation maps frequency rank r = 1..V to a token id (so surviving rows are
    scattered through W); rank r carries weight r**-s; ids are drawn without replacement with
    probability proportional to weight (exponential keys: keep the V_draft largest
    ln(u_r)/w_r).  V_draft == V gives the identity 0..V-1.
    """
    if not 0 < V_draft <= V:
        raise ValueError("need 0 < V_draft <= V")
    if V_draft == V:
        return np.arange(V, dtype=np.int32)
    perm = np.argsort(raw_u64(seed, STREAM_PERM, 0, V), kind="stable")
    w = np.arange(1, V + 1, dtype=np.float64) ** (-s)
    keys = np.log(uniform01(seed, STREAM_KEYS, 0, V)) / w
    chosen_ranks = np.argpartition(-keys, V_draft - 1)[:V_draft]
    return np.sort(perm[chosen_ranks]).astype(np.int32)


def zipf_token_stream(seed: int, V: int, n: int, s: float = 1.1, support: int | None = None) -> np.ndarray:
    """n token ids in [0,V), int32, drawn independently: frequency rank r = 1..support has
    probability proportional to r**-s and the same seeded permutation as zipf_subset maps
    ranks to ids (ranks beyond `support` never occur: tokens with zero frequency).  Stands in
    for the assistant-span token stream of a training corpus (Section 2.2)."""
    support = V if support is None else support
    if not 0 < support <= V or n < 0:
        raise ValueError("need 0 < support <= V and n >= 0")
    perm = np.argsort(raw_u64(seed, STREAM_PERM, 0, V), kind="stable")
    w = np.arange(1, support + 1, dtype=np.float64) ** (-s)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    out = np.empty(n, dtype=np.int32)
    step = 1 << 22
    for a in range(0, n, step):
        b = min(n, a + step)
        u = uniform01(seed, STREAM_TOKENS, a, b - a)
        r = np.minimum(np.searchsorted(cdf, u, side="right"), support - 1)
        out[a:b] = perm[r]
    return out


def small_int_bf16(seed: int, stream: int, shape, lo: int = -4, hi: int = 4) -> np.ndarray:
    """Small integers in [lo,hi] as bf16 bits (exactly representable): any-order fp32 sums of
    their products are exact while |sum| < 2**24."""
    n = int(np.prod(shape))
    span = np.uint64(hi - lo + 1)
    v = (raw_u64(seed, stream, 0, n) % span).astype(np.int64) + lo
    return f32_to_bf16(v.astype(np.float32)).reshape(shape)


# The five workload shapes the head is measured and tested on.
CONFIGS = {
    "cfg0": dict(H=2048, rows=(1,), V_draft=(4096,), k=1, peaked=0.0),
    "cfg1": dict(H=2048, rows=(1, 4, 8), V_draft=(FULL_VOCAB,), k=10, peaked=0.0),
    "cfg2": dict(H=4096, rows=(1,), V_draft=(4096, 8192, 16384, 32768, 65536, FULL_VOCAB), k=10, peaked=0.0),
    "cfg3": dict(H=4096, rows=(1024,), V_draft=(32000,), k=8, peaked=0.0),
    "cfg4": dict(H=4096, rows=(512,), V_draft=(FULL_VOCAB,), k=16, peaked=0.05),
}
