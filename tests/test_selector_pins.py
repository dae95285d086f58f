"""Pins for the vocabulary-size selection oracle (oracle/vs_oracle.py): each test ties it to a
fact outside itself -- values the paper prints for Eq. 3 with Table 1's numbers, closed forms
for simple frequency laws, exact rational arithmetic on tiny vocabularies, invariants of
Eq. 2-5, and plain library routines for the counting and ordering steps.
"""
import collections
from fractions import Fraction

import numpy as np
import pytest

from oracle import vs_oracle as vs
from paper_2603_05210_amd import synth


def _read_table1(golden_dir):
    vals = {}
    for line in (golden_dir / "table1_flops.txt").read_text().splitlines():
        if line.startswith("#") or not line.strip():
            continue
        parts = line.split()
        vals[parts[0]] = [float(x) for x in parts[1:]]
    return vals


def _stream_from_counts(counts, seed=0):
    """A token stream with exactly these frequencies, in a seeded shuffled order."""
    toks = np.repeat(np.arange(len(counts), dtype=np.int32), counts)
    order = np.argsort(synth.raw_u64(seed, synth.STREAM_KEYS, 0, toks.size), kind="stable")
    return toks[order]


# ------------------------------------------------ values printed in the paper (Eq. 3, Table 1)
def test_latency_reduction_matches_the_papers_printed_values(golden_dir):
    t = _read_table1(golden_dir)
    d, V = int(t["d"][0]), int(t["V"][0])
    F_fixed = (t["feature_fusion"][0] + t["attention"][0] + t["feed_forward"][0]) * 1e6
    # the head's own cost in the table is 2 d V
    assert abs(2.0 * d * V / 1e6 - t["lm_head"][0]) < 0.05
    R = vs.latency_reduction(np.array([13264, 1, V]), d, V, F_fixed)
    assert abs(100.0 * R[0] - t["R_at_13264"][0]) < 0.05     # 57.5 % at the selected size
    assert round(100.0 * R[1]) == t["R_max"][0]               # the largest reduction the paper quotes
    assert R[2] == 0.0                                         # the full vocabulary saves nothing
    # the head's share of the draft's FLOPs is the limit of R as k -> 0 (64.15 from the table's
    # own rounded entries, printed as 64.2)
    assert abs(100.0 * vs.latency_reduction(np.array([0]), d, V, F_fixed)[0] - t["lm_head"][1]) < 0.06


def test_a_dropped_factor_or_a_flipped_ratio_would_miss_the_printed_value(golden_dir):
    t = _read_table1(golden_dir)
    d, V = int(t["d"][0]), int(t["V"][0])
    F = (t["feature_fusion"][0] + t["attention"][0] + t["feed_forward"][0]) * 1e6
    k = 13264.0
    wrong = [1 - (F + d * k) / (F + d * V),            # head cost d k instead of 2 d k
             1 - (2 * d * k) / (2 * d * V),            # fixed cost left out
             (F + 2 * d * k) / (F + 2 * d * V),        # the ratio instead of the reduction
             1 - (F + 2 * d * k) / (2 * d * V)]        # fixed cost missing from the denominator
    for w in wrong:
        assert abs(100.0 * w - t["R_at_13264"][0]) > 0.5


# ------------------------------------------------ closed forms
@pytest.mark.parametrize("alpha,expect", [(0.9, "k_max"), (0.1, "k_min")])
def test_uniform_frequencies_make_utility_linear(alpha, expect):
    V, d, F = 500, 64, 3.0e4
    s = vs.select_vocab(_stream_from_counts(np.full(V, 7)), V, d, F, alpha, 0.0, 10, 400)
    k = np.arange(V + 1)
    assert np.array_equal(s.curve_C, k / V)                     # C(k) = k / V exactly
    slope = alpha / V - (1 - alpha) * 2 * d / (F + 2 * d * V)   # dU/dk, constant
    assert (slope > 0) == (expect == "k_max")
    assert s.k_star == (400 if expect == "k_max" else 10)
    assert np.array_equal(s.rank_ids, np.arange(V))             # all equal: id order


def test_two_level_frequencies_peak_at_the_kink():
    V, d, F, m, A, B = 300, 32, 1.0e4, 40, 50, 1
    counts = np.full(V, B)
    hot = np.arange(V)[::7][:m]                                 # the m frequent ids, scattered
    counts[hot] = A
    T = counts.sum()
    den = F + 2 * d * V
    # alpha with slope A*alpha/T - (1-alpha)*2d/den > 0 on the hot part and < 0 on the tail
    lo = (2 * d / den) / (A / T + 2 * d / den)
    hi = (2 * d / den) / (B / T + 2 * d / den)
    alpha = 0.5 * (lo + hi)
    s = vs.select_vocab(_stream_from_counts(counts, 1), V, d, F, alpha, 0.0, 1, V)
    assert s.k_star == m
    assert np.array_equal(np.sort(s.rank_ids[:m]), np.sort(hot))
    assert np.array_equal(s.token_ids, np.sort(hot).astype(np.int32))
    assert abs(s.C - m * A / T) < 1e-15


# ------------------------------------------------ exact rational arithmetic on tiny inputs
@pytest.mark.parametrize("seed", range(8))
def test_argmax_equals_exact_rational_argmax(seed):
    V = 12
    counts = (synth.raw_u64(seed, synth.STREAM_KEYS, 100, V) % np.uint64(9)).astype(np.int64)
    counts[int(seed) % V] += 1                                  # never an empty stream
    d, F = 5, 137
    alpha = Fraction(1 + seed, 10)
    c_min = Fraction(seed % 4, 5)
    k_min, k_max = 1 + seed % 3, V - seed % 2
    order = sorted(range(V), key=lambda v: (-int(counts[v]), v))
    T = int(counts.sum())
    best, best_k = None, None
    pre = 0
    for k in range(0, V + 1):
        if k > 0:
            pre += int(counts[order[k - 1]])
        C = Fraction(pre, T)
        R = 1 - Fraction(F + 2 * d * k, F + 2 * d * V)
        U = alpha * C + (1 - alpha) * R if C >= c_min else Fraction(-1)
        if k_min <= k <= k_max and (best is None or U > best):
            best, best_k = U, k
    s = vs.select_vocab(_stream_from_counts(counts, seed), V, d, float(F), float(alpha), float(c_min), k_min, k_max)
    assert s.k_star == best_k
    assert list(s.rank_ids) == order
    if best >= 0:
        assert abs(s.U - float(best)) < 1e-14


# ------------------------------------------------ invariants of Eq. 2-5
def test_curves_are_monotone_and_normalised():
    V = 5000
    toks = synth.zipf_token_stream(3, V, 200_000, support=3000)
    s = vs.select_vocab(toks, V, 128, 5.0e5, 0.5, 0.0, 1, V)
    C = s.curve_C
    assert C[0] == 0.0 and C[V] == 1.0
    assert np.all(np.diff(C) >= 0.0)
    assert np.all(np.diff(np.diff(C)) <= 1e-15)                 # concave: frequencies descend
    k = np.arange(V + 1)
    R = vs.latency_reduction(k, 128, V, 5.0e5)
    assert np.all(np.diff(R) < 0.0) and R[V] == 0.0
    f_sorted = s.f[s.rank_ids]
    assert np.all(np.diff(f_sorted) <= 0)
    assert np.all(s.f[s.rank_ids[3000:]] == 0)                  # the unseen tokens come last ...
    assert np.all(np.diff(s.rank_ids[np.flatnonzero(f_sorted == 0)]) > 0)  # ... in id order


def test_counting_and_ordering_match_plain_python():
    V = 97
    toks = synth.zipf_token_stream(5, V, 4000)
    f = vs.token_frequencies(toks, V)
    ctr = collections.Counter(int(t) for t in toks)
    assert all(int(f[v]) == ctr.get(v, 0) for v in range(V)) and int(f.sum()) == 4000
    assert list(vs.rank_by_frequency(f)) == sorted(range(V), key=lambda v: (-ctr.get(v, 0), v))


def test_stream_order_does_not_matter_and_relabelling_commutes():
    V = 400
    toks = synth.zipf_token_stream(7, V, 50_000)
    a = vs.select_vocab(toks, V, 64, 2.0e4, 0.6, 0.5, 1, V)
    b = vs.select_vocab(toks[::-1].copy(), V, 64, 2.0e4, 0.6, 0.5, 1, V)
    assert a.k_star == b.k_star and np.array_equal(a.rank_ids, b.rank_ids)
    relabel = np.argsort(synth.raw_u64(9, synth.STREAM_PERM, 0, V), kind="stable").astype(np.int32)
    c = vs.select_vocab(relabel[toks], V, 64, 2.0e4, 0.6, 0.5, 1, V)
    assert c.k_star == a.k_star and c.C == a.C
    # the selected SET is the relabelled set wherever frequencies are distinct at the boundary
    fa = a.f[a.rank_ids]
    if fa[a.k_star - 1] != fa[a.k_star]:
        assert np.array_equal(np.sort(relabel[a.rank_ids[:a.k_star]]), c.token_ids)


# ------------------------------------------------ the coverage constraint (Eq. 5)
def test_coverage_constraint_bounds_the_choice_from_below():
    V = 2000
    toks = synth.zipf_token_stream(11, V, 100_000)
    free = vs.select_vocab(toks, V, 256, 1.0e5, 0.0, 0.0, 1, V)
    assert free.k_star == 1                                      # alpha = 0: pure latency
    c_min = 0.9
    s = vs.select_vocab(toks, V, 256, 1.0e5, 0.0, c_min, 1, V)
    k_c = int(np.argmax(s.curve_C >= c_min))                     # smallest k meeting the constraint
    assert s.feasible and s.k_star == k_c and s.curve_C[k_c - 1] < c_min <= s.C
    assert np.all(s.curve_U[:k_c] == -1.0)
    t = vs.select_vocab(toks, V, 256, 1.0e5, 0.0, c_min, 1, k_c - 1)
    assert not t.feasible and t.k_star == 1                      # nothing feasible: first k of the range
    assert np.array_equal(s.token_ids, np.sort(s.rank_ids[:k_c]))


def test_bad_arguments_are_rejected():
    with pytest.raises(ValueError):
        vs.select_vocab(np.array([0, 5], dtype=np.int32), 5, 8, 1.0, 0.5, 0.0, 1, 5)
    with pytest.raises(ValueError):
        vs.select_vocab(np.array([], dtype=np.int32), 5, 8, 1.0, 0.5, 0.0, 1, 5)
    with pytest.raises(ValueError):
        vs.select_vocab(np.array([1], dtype=np.int32), 5, 8, 1.0, 0.5, 0.0, 0, 5)
