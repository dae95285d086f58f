"""Pins for the coverage / t2d oracle (oracle/vc_oracle.py): the paper's Table 4 (the combined
row is the occurrence-weighted combination of the benchmark rows), the selector oracle's C(k)
on the same stream (Eq. 2), closed forms, and plain Python set arithmetic."""
import numpy as np
import pytest

from oracle import vc_oracle as vc
from oracle import vs_oracle as vs
from paper_2603_05210_amd import synth


def test_combined_row_of_table4_is_the_occurrence_weighted_combination(golden_dir):
    rows = []
    for line in (golden_dir / "table4_coverage.txt").read_text().splitlines():
        if line.startswith("#") or not line.strip():
            continue
        name, n, fc, uc = line.split()
        rows.append((name, int(n), float(fc)))
    parts = [vc.Coverage(n, round(n * fc / 100.0), 1, 1, fc / 100.0, 1.0, np.zeros(0, np.int32))
             for name, n, fc in rows if name != "Combined"]
    n, c, f = vc.combine(parts)
    comb = [r for r in rows if r[0] == "Combined"][0]
    assert n == comb[1]                                 # 574,168 generated tokens in all
    assert abs(100.0 * f - comb[2]) < 0.06              # 97.1 %
    # an unweighted mean of the rows would print 96.4, not 97.1
    assert abs(np.mean([fc for name, _, fc in rows if name != "Combined"]) - comb[2]) > 0.5


def test_frequency_coverage_of_the_top_k_equals_eq2_on_the_same_stream():
    V = 3000
    toks = synth.zipf_token_stream(1, V, 150_000)
    sel = vs.select_vocab(toks, V, 128, 5.0e5, 0.5, 0.9, 1, V)
    t2d = vc.build_t2d(sel.token_ids, V)
    cov = vc.coverage(toks, t2d)
    assert cov.freq_coverage == sel.C                   # the same ratio of the same integers
    assert cov.n_covered == int(sel.f[sel.rank_ids[:sel.k_star]].sum())
    assert cov.n_unique == int(np.count_nonzero(sel.f))
    # another stream of the same law: rare tokens are the uncovered ones, so the share of
    # distinct tokens covered stays below the share of occurrences covered (Table 4's pattern)
    other = vc.coverage(synth.zipf_token_stream(2, V, 50_000), t2d)
    assert 0.0 < other.unique_coverage < other.freq_coverage <= 1.0


def test_t2d_inverts_d2t():
    V = 500
    d2t = synth.zipf_subset(3, V, 120)
    t2d = vc.build_t2d(d2t, V)
    assert np.array_equal(t2d[d2t], np.arange(120))
    assert np.count_nonzero(t2d >= 0) == 120 and np.all(t2d[np.setdiff1d(np.arange(V), d2t)] == -1)
    # unsorted draft order is kept: the draft index is the position in the list
    perm = d2t[::-1].copy()
    assert np.array_equal(vc.build_t2d(perm, V)[perm], np.arange(120))
    with pytest.raises(ValueError):
        vc.build_t2d(np.array([1, 1]), V)
    with pytest.raises(ValueError):
        vc.build_t2d(np.array([V]), V)


def test_closed_forms_and_set_arithmetic():
    V = 50
    toks = np.array([3, 3, 3, 7, 7, 9, 11, 11, 11, 11], dtype=np.int32)
    t2d = vc.build_t2d(np.array([11, 3, 40]), V)
    c = vc.coverage(toks, t2d)
    assert (c.n_tokens, c.n_covered, c.n_unique, c.n_unique_covered) == (10, 7, 4, 2)
    assert c.freq_coverage == 0.7 and c.unique_coverage == 0.5
    assert list(c.draft_ids) == [1, 1, 1, -1, -1, -1, 0, 0, 0, 0]
    # every seen token in the vocabulary -> both coverages 1; none -> 0
    assert vc.coverage(toks, vc.build_t2d(np.array([3, 7, 9, 11]), V)).unique_coverage == 1.0
    none = vc.coverage(toks, vc.build_t2d(np.array([0, 1, 2]), V))
    assert none.freq_coverage == 0.0 and none.unique_coverage == 0.0
    # plain Python
    toks2 = synth.zipf_token_stream(5, 400, 5000)
    d2t = synth.zipf_subset(5, 400, 60)
    c2 = vc.coverage(toks2, vc.build_t2d(d2t, 400))
    S = set(int(x) for x in d2t)
    assert c2.n_covered == sum(1 for t in toks2 if int(t) in S)
    assert c2.n_unique_covered == len(set(int(t) for t in toks2) & S)
