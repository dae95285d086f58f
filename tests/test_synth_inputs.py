"""The seeded input generators: reproducible, sliceable, and shaped as stated."""
import numpy as np
import torch

from paper_2603_05210_amd import synth


def test_bf16_rounding_matches_torch_round_to_nearest_even():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000).astype(np.float32) * 3,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 65280.0, 1e-30], dtype=np.float32)])
    ours = synth.f32_to_bf16(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, ref)
    back = synth.bf16_to_f32(ours)
    assert np.array_equal(back, torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_streams_are_counter_based_and_reproducible():
    a = synth.normal(0, 0, 0, 1001)
    b = np.concatenate([synth.normal(0, 0, 0, 333), synth.normal(0, 0, 333, 668)])
    assert np.array_equal(a, b)
    assert not np.array_equal(a, synth.normal(1, 0, 0, 1001))
    assert not np.array_equal(a, synth.normal(0, 1, 0, 1001))
    W = synth.gen_W(0, 700, 64)
    assert np.array_equal(W[100:130], synth.gen_W(0, 700, 64, row0=100, row1=130))
    assert np.array_equal(W[[5, 699, 13]], synth.gen_W_rows(0, 64, [5, 699, 13]))


def test_distributions():
    x = synth.normal(0, 0, 0, 400000)
    assert abs(x.mean()) < 0.01 and abs(x.std() - 1.0) < 0.01
    assert abs(np.mean(x ** 4) - 3.0) < 0.1
    W = synth.bf16_to_f32(synth.gen_W(0, 2000, 128, 0.02))
    assert abs(W.std() - 0.02) < 5e-4
    h = synth.bf16_to_f32(synth.gen_h(0, 200, 256, peaked_frac=0.05))
    rows = synth.peaked_rows(0, 200, 0.05)
    assert len(rows) == 10
    rs = h.std(axis=1)
    mask = np.zeros(200, dtype=bool)
    mask[rows] = True
    assert np.all(rs[mask] > 7.0) and np.all(rs[~mask] < 1.5)


def test_zipf_subset_shape_and_bias():
    V = 20000
    ids = synth.zipf_subset(0, V, 2000)
    assert ids.dtype == np.int32 and len(ids) == 2000
    assert np.all(np.diff(ids) > 0) and ids[0] >= 0 and ids[-1] < V
    assert np.array_equal(synth.zipf_subset(0, V, V), np.arange(V, dtype=np.int32))
    # frequent ranks survive far more often than rare ones
    perm = np.argsort(synth.raw_u64(0, synth.STREAM_PERM, 0, V), kind="stable")
    rank_of = np.empty(V, dtype=np.int64)
    rank_of[perm] = np.arange(V)
    ranks = rank_of[ids]
    assert np.mean(ranks < 2000) > 0.5
    assert np.array_equal(ids, synth.zipf_subset(0, V, 2000))
    assert not np.array_equal(ids, synth.zipf_subset(1, V, 2000))


def test_token_stream_is_seeded_in_range_and_heavy_tailed():
    V, n = 3000, 300_000
    a = synth.zipf_token_stream(4, V, n)
    b = synth.zipf_token_stream(4, V, n)
    assert a.dtype == np.int32 and a.shape == (n,) and np.array_equal(a, b)
    assert a.min() >= 0 and a.max() < V
    # a prefix of a longer stream is the shorter stream (counter-based draws)
    assert np.array_equal(synth.zipf_token_stream(4, V, 1000), a[:1000])
    f = np.sort(np.bincount(a, minlength=V))[::-1]
    assert f[0] > 20 * f[V // 10]                    # Zipf(1.1): the head dominates
    # restricted support: exactly `support` ids can occur
    c = synth.zipf_token_stream(4, V, n, support=100)
    assert np.unique(c).size <= 100
    assert not np.array_equal(synth.zipf_token_stream(5, V, 1000), a[:1000])
