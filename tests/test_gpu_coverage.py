"""GPU parity of the target-to-draft buffer and the coverage measurements against
oracle/vc_oracle.py: integer work, compared for equality (the two ratios are one double
division of those integers on each side)."""
import numpy as np
import pytest
import torch

import paper_2603_05210_amd as vt
from oracle import vc_oracle as vc
from oracle import vs_oracle as vs
from paper_2603_05210_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _check(tokens, d2t, V):
    t2d_dev = vt.vt_build_t2d(_dev(d2t), V)
    t2d_o = vc.build_t2d(d2t, V)
    assert np.array_equal(t2d_dev.cpu().numpy(), t2d_o), "t2d differs"
    res, draft = vt.vt_coverage(_dev(tokens), t2d_dev, want_draft_ids=True)
    ora = vc.coverage(tokens, t2d_o)
    got = (int(res.n_tokens), int(res.n_covered), int(res.n_unique), int(res.n_unique_covered))
    assert got == (ora.n_tokens, ora.n_covered, ora.n_unique, ora.n_unique_covered), (got, ora)
    assert res.freq_coverage == ora.freq_coverage and res.unique_coverage == ora.unique_coverage
    assert np.array_equal(draft.cpu().numpy(), ora.draft_ids), "mapped stream differs"
    res2, none = vt.vt_coverage(_dev(tokens), t2d_dev)          # without the mapped stream
    assert none is None
    got2 = (int(res2.n_tokens), int(res2.n_covered), int(res2.n_unique), int(res2.n_unique_covered))
    assert got2 == got and res2.freq_coverage == ora.freq_coverage and res2.unique_coverage == ora.unique_coverage
    return res, ora


@pytest.mark.parametrize("V,Vd,n,support", [
    (50, 3, 10, 50),
    (400, 60, 5000, 400),
    (5000, 700, 300_001, 3000),
    (128256, 13264, 2_000_000, 128256),   # the paper's vocabulary and its selected size
    (128256, 128256, 500_000, 128256),    # the full vocabulary covers everything
    (128256, 4380, 3_000_001, 90_000),    # long stream: the ratios-only call keeps its bitmaps in LDS
    (300_000, 20_000, 1_500_000, 300_000),  # long stream, vocabulary a little too wide for that
    (1000, 1, 10_000, 1000),
])
def test_coverage_matches_oracle(V, Vd, n, support):
    print("coverage V=%d Vd=%d n=%d" % (V, Vd, n), flush=True)
    tokens = synth.zipf_token_stream(V + Vd, V, n, support=support)
    d2t = synth.zipf_subset(V + Vd, V, Vd)
    res, ora = _check(tokens, d2t, V)
    if Vd == V:
        assert res.freq_coverage == 1.0 and res.unique_coverage == 1.0


@pytest.mark.parametrize("skip", [1, 2, 3])
def test_long_stream_that_starts_off_a_16_byte_boundary(skip):
    """The ratios-only call reads the stream with 16-byte loads over its aligned middle: a stream that
    starts 4, 8 or 12 bytes past a boundary (and ends raggedly) gives the oracle's counts all the same."""
    V, Vd, n = 128256, 6521, 1_200_003
    tokens = synth.zipf_token_stream(11, V, n + skip)
    d2t = synth.zipf_subset(11, V, Vd)
    t2d_dev = vt.vt_build_t2d(_dev(d2t), V)
    view = _dev(tokens)[skip:]
    assert view.data_ptr() % 16 == 4 * skip
    res, none = vt.vt_coverage(view, t2d_dev)
    ora = vc.coverage(tokens[skip:], vc.build_t2d(d2t, V))
    got = (int(res.n_tokens), int(res.n_covered), int(res.n_unique), int(res.n_unique_covered))
    assert got == (ora.n_tokens, ora.n_covered, ora.n_unique, ora.n_unique_covered), (got, ora)


def test_unsorted_draft_order_is_kept():
    V = 300
    d2t = synth.zipf_subset(1, V, 40)[::-1].copy()
    _check(synth.zipf_token_stream(1, V, 3000), d2t, V)


def test_selected_vocabulary_reaches_its_own_coverage():
    """select -> build_subset -> t2d -> coverage on the stream the vocabulary was selected from
    gives C(k*) exactly (Eq. 2)."""
    V, H = 4000, 64
    tokens = synth.zipf_token_stream(9, V, 250_000)
    t_dev = _dev(tokens)
    sel, _, _, ids = vt.vt_select_vocab(t_dev, V, H, 1.0e5, 0.5, 0.9, 16, V)
    W_dev = torch.from_numpy(synth.gen_W(9, V, H).view(np.int16)).to(DEV)
    _, d2t = vt.vt_build_subset(W_dev, ids.contiguous())
    t2d = vt.vt_build_t2d(d2t, V)
    res, _ = vt.vt_coverage(t_dev, t2d)
    assert res.freq_coverage == sel.C
    ora = vs.select_vocab(tokens, V, H, 1.0e5, 0.5, 0.9, 16, V)
    assert res.freq_coverage == ora.C and int(res.n_unique_covered) == ora.k_star


def test_bad_ids_are_reported():
    V = 100
    with pytest.raises(vt.VtError) as e:
        vt.vt_build_t2d(_dev(np.array([5, 7, 5], dtype=np.int32)), V)
    assert e.value.status == 5
    with pytest.raises(vt.VtError) as e:
        vt.vt_build_t2d(_dev(np.array([5, 100], dtype=np.int32)), V)
    assert e.value.status == 4
    t2d = vt.vt_build_t2d(_dev(np.array([5, 7], dtype=np.int32)), V)
    with pytest.raises(vt.VtError) as e:
        vt.vt_coverage(_dev(np.array([5, -1, 7], dtype=np.int32)), t2d)
    assert e.value.status == 4


def test_workspace_is_reusable():
    V = 2000
    ws = torch.empty(vt.vt_coverage_workspace_bytes(V), dtype=torch.uint8, device=DEV)
    d2t = synth.zipf_subset(2, V, 300)
    t2d = vt.vt_build_t2d(_dev(d2t), V, workspace=ws)
    t2d_o = vc.build_t2d(d2t, V)
    for seed, n in ((1, 50_000), (2, 999), (1, 50_000)):
        toks = synth.zipf_token_stream(seed, V, n)
        res, _ = vt.vt_coverage(_dev(toks), t2d, workspace=ws)
        ora = vc.coverage(toks, t2d_o)
        assert (int(res.n_covered), int(res.n_unique), int(res.n_unique_covered)) == \
            (ora.n_covered, ora.n_unique, ora.n_unique_covered)
