"""TEST INFRASTRUCTURE -- CPU oracle of the target-to-draft index buffer and of the token
coverage measurements (Section 1: the t2d / d2t buffers; Section 2.2, Eq. 2 and Section 5.1,
Table 4: frequency-weighted and unique coverage of a draft vocabulary on a token stream).
Plain numpy, integers only until the two final ratios.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this module; the
product package never does, and this module imports nothing from the product.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


def build_t2d(d2t: np.ndarray, V: int) -> np.ndarray:
    """t2d[v] = j where d2t[j] = v, and -1 for every target token outside the draft vocabulary
    (Section 1: the inverse of the draft-to-target buffer).  int32[V]."""
    d2t = np.asarray(d2t, dtype=np.int64)
    if d2t.size and (d2t.min() < 0 or d2t.max() >= V):
        raise ValueError("draft-to-target id outside [0,V)")
    if np.unique(d2t).size != d2t.size:
        raise ValueError("draft-to-target ids repeat")
    t2d = np.full(V, -1, dtype=np.int32)
    t2d[d2t] = np.arange(d2t.size, dtype=np.int32)
    return t2d


@dataclass
class Coverage:
    n_tokens: int            # occurrences in the stream
    n_covered: int           # occurrences whose token is in the draft vocabulary
    n_unique: int            # distinct tokens in the stream
    n_unique_covered: int    # distinct tokens in the stream that are in the draft vocabulary
    freq_coverage: float     # n_covered / n_tokens          (Table 4, frequency-weighted column; Eq. 2 on this stream)
    unique_coverage: float   # n_unique_covered / n_unique   (Table 4, unique-token column)
    draft_ids: np.ndarray    # int32[n]: t2d[token], -1 where the target token has no draft index


def coverage(tokens: np.ndarray, t2d: np.ndarray) -> Coverage:
    tokens = np.asarray(tokens, dtype=np.int64)
    V = t2d.shape[0]
    if tokens.size == 0:
        raise ValueError("empty token stream")
    if tokens.min() < 0 or tokens.max() >= V:
        raise ValueError("token id outside [0,V)")
    draft_ids = t2d[tokens].astype(np.int32)
    n = int(tokens.size)
    n_cov = int(np.count_nonzero(draft_ids >= 0))
    distinct = np.unique(tokens)
    n_uni = int(distinct.size)
    n_uni_cov = int(np.count_nonzero(t2d[distinct] >= 0))
    return Coverage(n, n_cov, n_uni, n_uni_cov, n_cov / n, n_uni_cov / n_uni, draft_ids)


def combine(parts) -> tuple[int, int, float]:
    """Coverage of several streams taken together: occurrences add up (the combined row of Table 4)."""
    n = sum(p.n_tokens for p in parts)
    c = sum(p.n_covered for p in parts)
    return n, c, c / n
