"""GPU parity of the vocabulary-size selection (Eq. 1-5) against oracle/vs_oracle.py.

Integer results (frequencies, ranking, k*, the selected ids) must be identical; C, R and U at
k* are IEEE doubles computed by the same operations in the same order on both sides, so they
must be identical too.
"""
import numpy as np
import pytest
import torch

import paper_2603_05210_amd as vt
from oracle import vs_oracle as vs
from paper_2603_05210_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

# Table 1 of the paper: the draft's FLOPs that do not depend on the vocabulary, d and V
F_FIXED = (100.7 + 436.2 + 50.3) * 1e6
D_PAPER, V_PAPER = 4096, 128256


def _say(msg):
    print(msg, flush=True)


def _run_both(tokens, V, d, F, alpha, c_min, k_min, k_max):
    t_dev = torch.from_numpy(tokens).to(DEV)
    res, freq, rank_ids, token_ids = vt.vt_select_vocab(t_dev, V, d, F, alpha, c_min, k_min, k_max)
    torch.cuda.synchronize()
    ora = vs.select_vocab(tokens, V, d, F, alpha, c_min, k_min, k_max)
    assert np.array_equal(freq.cpu().numpy().view(np.uint32).astype(np.int64), ora.f), "frequencies differ"
    assert np.array_equal(rank_ids.cpu().numpy(), ora.rank_ids), "ranking differs"
    assert int(res.k_star) == ora.k_star, "k* differs: %d vs %d" % (res.k_star, ora.k_star)
    assert bool(res.feasible) == ora.feasible
    assert int(res.n_tokens) == tokens.size
    assert np.array_equal(token_ids.cpu().numpy(), ora.token_ids), "selected ids differ"
    assert res.C == ora.C and res.R == ora.R and res.U == ora.U, "C/R/U differ in some bit"
    return res, ora


CASES = [
    # V, n, support, d, F, alpha, c_min, k_min, k_max
    (12, 50, 12, 5, 137.0, 0.3, 0.0, 1, 12),
    (12, 3, 5, 5, 137.0, 0.5, 0.2, 2, 11),                 # fewer tokens than one vector load
    (1000, 100_003, 1000, 64, 2.0e4, 0.6, 0.5, 1, 1000),    # stream length not a multiple of 4
    (5000, 400_000, 3000, 128, 5.0e5, 0.5, 0.9, 100, 4000),  # 2000 tokens never occur
    (4096, 50_000, 4096, 32, 1.0e4, 0.2, 0.0, 1, 4096),     # exactly one sort chunk
    (4097, 60_000, 4097, 32, 1.0e4, 0.8, 0.95, 1, 4097),    # one key past a sort chunk
    (70_000, 1_000_000, 70_000, 2048, 3.0e8, 0.5, 0.9, 1024, 70_000),
    (2000, 100_000, 2000, 256, 1.0e5, 0.0, 0.9, 1, 2000),   # alpha = 0: the constraint decides
    (2000, 100_000, 2000, 256, 1.0e5, 1.0, 0.0, 1, 1500),   # alpha = 1: coverage only -> k_max
    (2000, 100_000, 2000, 256, 1.0e5, 0.5, 0.999999, 1, 50),  # nothing feasible in the range
    (2000, 100_000, 2000, 256, 1.0e5, 0.5, 0.5, 700, 700),  # a single candidate
]


@pytest.mark.parametrize("V,n,support,d,F,alpha,c_min,k_min,k_max", CASES)
def test_selection_matches_oracle(V, n, support, d, F, alpha, c_min, k_min, k_max):
    _say("select V=%d n=%d support=%d alpha=%g c_min=%g range=[%d,%d]" % (V, n, support, alpha, c_min, k_min, k_max))
    tokens = synth.zipf_token_stream(V + n, V, n, support=support)
    res, ora = _run_both(tokens, V, d, F, alpha, c_min, k_min, k_max)
    _say("  k*=%d C=%.6f R=%.6f U=%.6f feasible=%d" % (res.k_star, res.C, res.R, res.U, res.feasible))


def test_all_frequencies_equal_orders_by_id():
    V = 6000
    tokens = np.repeat(np.arange(V, dtype=np.int32), 3)
    tokens = tokens[np.argsort(synth.raw_u64(1, synth.STREAM_KEYS, 0, tokens.size), kind="stable")]
    res, ora = _run_both(tokens, V, 64, 3.0e4, 0.9, 0.0, 10, 5000)
    assert res.k_star == 5000 and np.array_equal(ora.rank_ids, np.arange(V))


@pytest.mark.parametrize("alpha,c_min", [(0.5, 0.9), (0.3, 0.937), (0.7, 0.0)])
def test_paper_sized_selection(alpha, c_min):
    """LLaMA-3's vocabulary and Table 1's constants on a Zipf(1.1) stream of 8 M tokens."""
    _say("select paper-sized alpha=%g c_min=%g" % (alpha, c_min))
    tokens = synth.zipf_token_stream(0, V_PAPER, 8_000_000)
    res, ora = _run_both(tokens, V_PAPER, D_PAPER, F_FIXED, alpha, c_min, 1024, V_PAPER)
    _say("  k*=%d C=%.4f R=%.4f U=%.4f" % (res.k_star, res.C, res.R, res.U))
    # the selected ids feed the head's set-up call as they are
    assert vt.vt_check_token_ids_host(ora.token_ids, V_PAPER) == vt.VT_OK


def test_selection_at_the_benchmarked_size():
    """The configuration bench.py times: 32 Mi tokens over LLaMA-3's vocabulary."""
    _say("select at the benchmarked size")
    tokens = synth.zipf_token_stream(0, V_PAPER, 32 * 1024 * 1024)
    res, ora = _run_both(tokens, V_PAPER, D_PAPER, F_FIXED, 0.5, 0.9, 1024, V_PAPER)
    _say("  k*=%d C=%.4f R=%.4f U=%.4f" % (res.k_star, res.C, res.R, res.U))


def test_selected_ids_build_a_subset():
    V, H = 3000, 64
    tokens = synth.zipf_token_stream(2, V, 200_000)
    t_dev = torch.from_numpy(tokens).to(DEV)
    res, _, _, token_ids = vt.vt_select_vocab(t_dev, V, H, 1.0e4, 0.5, 0.9, 16, V)
    W = synth.gen_W(2, V, H)
    W_dev = torch.from_numpy(W.view(np.int16)).to(DEV)
    W_sub, d2t = vt.vt_build_subset(W_dev, token_ids.contiguous())
    torch.cuda.synchronize()
    ids = token_ids.cpu().numpy()
    assert np.array_equal(d2t.cpu().numpy(), ids)
    assert np.array_equal(W_sub.cpu().numpy().view(np.uint16), W[ids])


def test_out_of_range_token_is_reported():
    tokens = synth.zipf_token_stream(3, 500, 10_000)
    tokens[1234] = 500
    with pytest.raises(vt.VtError) as e:
        vt.vt_select_vocab(torch.from_numpy(tokens).to(DEV), 500, 64, 1.0e4, 0.5, 0.0, 1, 500)
    assert e.value.status == 4
    tokens[1234] = -1
    with pytest.raises(vt.VtError) as e:
        vt.vt_select_vocab(torch.from_numpy(tokens).to(DEV), 500, 64, 1.0e4, 0.5, 0.0, 1, 500)
    assert e.value.status == 4


@pytest.mark.parametrize("V,n", [(70_000, 1_500_001), (40_000, 1_048_576), (32_768, 2_000_003), (200_000, 1_200_000)])
def test_long_stream_histogram_by_id_classes(V, n):
    """Streams of a million tokens and more are counted per class of 32768 ids in plain LDS histograms:
    frequencies equal the oracle's for 1..7 classes and a ragged stream end, and ids outside [0, V) anywhere
    in the stream are reported."""
    _say("long stream V=%d n=%d" % (V, n))
    tokens = synth.zipf_token_stream(V + 7, V, n)
    res, freq, rank_ids, token_ids = vt.vt_select_vocab(torch.from_numpy(tokens).to(DEV), V, 256, 1.0e6, 0.5, 0.5, 1, V)
    assert np.array_equal(freq.cpu().numpy(), vs.token_frequencies(tokens, V))
    for pos, bad in ((n - 1, V), (n // 2 + 1, -3), (5, V + 40_000)):
        t2 = tokens.copy()
        t2[pos] = bad
        with pytest.raises(vt.VtError) as e:
            vt.vt_select_vocab(torch.from_numpy(t2).to(DEV), V, 256, 1.0e6, 0.5, 0.5, 1, V)
        assert e.value.status == 4


def test_repeated_calls_reuse_the_workspace():
    V = 9000
    ws = torch.empty(vt.vt_select_vocab_workspace_bytes(V), dtype=torch.uint8, device=DEV)
    a = synth.zipf_token_stream(4, V, 300_000)
    b = synth.zipf_token_stream(5, V, 100_000, support=500)
    for toks in (a, b, a):
        res, freq, rank_ids, token_ids = vt.vt_select_vocab(torch.from_numpy(toks).to(DEV), V, 128, 5.0e5, 0.5, 0.8,
                                                            1, V, workspace=ws)
        ora = vs.select_vocab(toks, V, 128, 5.0e5, 0.5, 0.8, 1, V)
        assert res.k_star == ora.k_star and np.array_equal(token_ids.cpu().numpy(), ora.token_ids)
