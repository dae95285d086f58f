"""TEST INFRASTRUCTURE -- CPU oracle of the draft-vocabulary size selection (Section 2 of the
paper: Eq. 1-5).  Plain numpy, float64, one function per equation, no blocking or fusion.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this module; the
product package never does, and this module imports nothing from the product.

What is computed, in the paper's notation:
  f(v)   token frequencies over a stream of token ids                      (Section 2.2)
  top-k  the k most frequent tokens; equal frequencies: lower token id first (reading)
  C(k)   = sum_{v in top-k} f(v) / sum_v f(v)                               (Eq. 2)
  R(k)   = 1 - (F_fixed + 2 d k) / (F_fixed + 2 d V)                        (Eq. 3)
  U(k)   = alpha C(k) + (1 - alpha) R(k)                                    (Eq. 4)
  U~(k)  = U(k) if C(k) >= c_min else -1                                    (Eq. 5)
  k*     = argmax_{k in [k_min, k_max]} U~(k)                               (Eq. 1)
The paper searches k with 100 TPE samples (Section 2.5); the arg-max over every k in the
range is the quantity that search approximates and is what is computed here.  Among equal
utilities the smallest k wins (reading: the paper does not say).

Floating point: every operation is a separate IEEE double operation in the order written
below (numpy never contracts a multiply and an add), so that another implementation doing the
same operations in the same order gets the same bits and therefore the same arg-max.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


def token_frequencies(tokens: np.ndarray, V: int) -> np.ndarray:
    """f(v) for v in [0,V): occurrences of each id in the stream (Section 2.2).  int64[V]."""
    tokens = np.asarray(tokens)
    if tokens.size and (tokens.min() < 0 or tokens.max() >= V):
        raise ValueError("token id outside [0,V)")
    return np.bincount(tokens.astype(np.int64), minlength=V).astype(np.int64)


def rank_by_frequency(f: np.ndarray) -> np.ndarray:
    """Token ids ordered by frequency, most frequent first; equal frequencies by lower id.
    rank_ids[:k] is the paper's top-k (Section 2.1).  int32[V]."""
    ids = np.arange(f.shape[0], dtype=np.int64)
    order = np.lexsort((ids, -f.astype(np.int64)))  # primary key -f, secondary key id
    return order.astype(np.int32)


def coverage(f: np.ndarray, rank_ids: np.ndarray) -> np.ndarray:
    """C(k) for k = 0..V (Eq. 2); C[0] = 0, C[V] = 1.  float64[V+1]."""
    total = int(f.sum())
    if total <= 0:
        raise ValueError("empty token stream")
    prefix = np.concatenate(([0], np.cumsum(f[rank_ids].astype(np.int64))))
    return prefix.astype(np.float64) / np.float64(total)


def latency_reduction(k: np.ndarray, d: int, V: int, F_fixed: float) -> np.ndarray:
    """R(k) (Eq. 3) with the head costing 2 d k FLOPs (Section 2.3).  float64."""
    two_d = np.float64(2.0) * np.float64(d)
    num = np.float64(F_fixed) + two_d * np.asarray(k, dtype=np.float64)
    den = np.float64(F_fixed) + two_d * np.float64(V)
    return np.float64(1.0) - num / den


def utility(C: np.ndarray, R: np.ndarray, alpha: float) -> np.ndarray:
    """U(k) (Eq. 4)."""
    a = np.float64(alpha)
    return a * C + (np.float64(1.0) - a) * R


def penalised_utility(U: np.ndarray, C: np.ndarray, c_min: float) -> np.ndarray:
    """U~(k) (Eq. 5)."""
    return np.where(C >= np.float64(c_min), U, np.float64(-1.0))


@dataclass
class Selection:
    k_star: int
    feasible: bool            # some k in the range meets the coverage constraint
    C: float                  # C(k*), R(k*), U(k*)
    R: float
    U: float
    f: np.ndarray             # int64[V]
    rank_ids: np.ndarray      # int32[V], most frequent first
    token_ids: np.ndarray     # int32[k*], the selected ids in ascending order (the head's V_d)
    curve_C: np.ndarray       # float64[V+1]
    curve_U: np.ndarray       # float64[V+1], the penalised utility


def select_vocab(tokens: np.ndarray, V: int, d: int, F_fixed: float, alpha: float, c_min: float,
                 k_min: int, k_max: int) -> Selection:
    """Eq. 1 over every k in [k_min, k_max] (1 <= k_min <= k_max <= V)."""
    if not 1 <= k_min <= k_max <= V:
        raise ValueError("need 1 <= k_min <= k_max <= V")
    f = token_frequencies(tokens, V)
    rank_ids = rank_by_frequency(f)
    C = coverage(f, rank_ids)
    k = np.arange(V + 1, dtype=np.int64)
    R = latency_reduction(k, d, V, F_fixed)
    U = penalised_utility(utility(C, R, alpha), C, c_min)
    window = U[k_min:k_max + 1]
    k_star = int(k_min + np.argmax(window))  # first maximum: the smallest k among equals
    feasible = bool(np.any(C[k_min:k_max + 1] >= np.float64(c_min)))
    token_ids = np.sort(rank_ids[:k_star]).astype(np.int32)
    return Selection(k_star, feasible, float(C[k_star]), float(R[k_star]), float(utility(C, R, alpha)[k_star]),
                     f, rank_ids, token_ids, C, U)
