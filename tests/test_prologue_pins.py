"""Pins of the prologue oracle (oracle/vp_oracle.py): the paper's FLOP count for the fusion layer,
library routines, closed forms and invariants of the normalisation and of the path scores."""
from pathlib import Path

import numpy as np
import torch

from oracle import vp_oracle as vp
from oracle import vt_oracle as vo
from paper_2603_05210_amd import synth

GOLDEN = Path(__file__).resolve().parent / "golden" / "table1_flops.txt"


def _table1():
    out = {}
    for line in GOLDEN.read_text().splitlines():
        f = line.split("#")[0].split()
        if len(f) >= 2:
            out[f[0]] = float(f[1])
    return out


def test_fusion_flops_are_table_1s():
    t = _table1()
    d = 4096
    assert vp.fusion_flops(3 * d, d) == 2 * 3 * d * d == 100663296
    assert t["d"] == d
    assert abs(vp.fusion_flops(3 * d, d) / 1e6 - t["feature_fusion"]) < 0.05   # Table 1 prints 100.7 M


def test_feature_fusion_against_library_matmul_and_identity_blocks():
    R, d = 3, 64
    x = synth.gen_h(1, R, 3 * d)
    W = synth.gen_W(1, d, 3 * d, std=0.05)
    g = vp.feature_fusion(x, W)
    ref = synth.bf16_to_f32(x).astype(np.float64) @ synth.bf16_to_f32(W).astype(np.float64).T
    gf = synth.bf16_to_f32(g).astype(np.float64)
    assert np.max(np.abs(gf - ref) / (np.abs(ref) + 1e-3)) < 2.0 ** -8    # one bf16 rounding of an fp32 sum
    # [0 | I | 0]: the projection returns the middle feature unchanged
    Wi = np.zeros((d, 3 * d), dtype=np.float32)
    Wi[np.arange(d), d + np.arange(d)] = 1.0
    assert np.array_equal(vp.feature_fusion(x, synth.f32_to_bf16(Wi).reshape(d, 3 * d)), x[:, d:2 * d])


def test_rmsnorm_library_closed_forms_and_invariants():
    R, H, eps = 5, 512, 1e-5
    g = synth.gen_h(2, R, H, peaked_frac=0.4)
    gamma = synth.f32_to_bf16((1.0 + 0.1 * synth.normal(2, 7, 0, H)).astype(np.float32))
    h = vp.rmsnorm(g, gamma, eps)
    # the library's rms_norm in fp32, rounded to bf16: equal up to one bf16 unit where the fp32 product sits on a boundary
    ref = torch.nn.functional.rms_norm(torch.from_numpy(synth.bf16_to_f32(g)), (H,), torch.from_numpy(synth.bf16_to_f32(gamma)), eps)
    ref16 = synth.f32_to_bf16(ref.numpy())
    diff = np.abs(h.astype(np.int32) - ref16.astype(np.int32))
    assert diff.max() <= 1 and (diff != 0).mean() < 0.01
    # unit root-mean-square before gamma
    hf = synth.bf16_to_f32(h).astype(np.float64) / synth.bf16_to_f32(gamma).astype(np.float64)[None]
    assert np.allclose(np.sqrt(np.mean(hf ** 2, axis=1)), 1.0, atol=5e-3)
    # scaling the input by a power of two changes nothing (eps = 0: exact)
    g4 = synth.f32_to_bf16(synth.bf16_to_f32(g) * 4.0)
    assert np.array_equal(vp.rmsnorm(g4, gamma, 0.0), vp.rmsnorm(g, gamma, 0.0))
    # a constant row c with gamma = 1 and eps = 0 normalises to sign(c)
    c = synth.f32_to_bf16(np.full((1, H), -3.0, dtype=np.float32))
    one = synth.f32_to_bf16(np.ones(H, dtype=np.float32))
    assert np.all(synth.bf16_to_f32(vp.rmsnorm(c, one, 0.0)) == -1.0)


def test_path_scores_follow_the_chain_rule():
    V, H, R = 60, 64, 4
    W = synth.gen_W(3, V, H, std=0.3)
    g = synth.gen_h(3, R, H)
    gamma = synth.f32_to_bf16(np.ones(H, dtype=np.float32))
    d2t = np.arange(V, dtype=np.int32)[::-1].copy()
    parent = np.log(np.array([0.5, 0.25, 0.125, 1.0], dtype=np.float32))
    res, scores, h = vp.head_fused(g, gamma, 1e-6, W, d2t, V, parent)      # k = V: every child of every node
    # the children of a node share out the node's own probability
    assert np.allclose(np.exp(scores.astype(np.float64)).sum(axis=1), np.exp(parent.astype(np.float64)), rtol=1e-5)
    # the head saw the normalised state, and no parent means the plain log-probabilities
    assert np.array_equal(res.ids, vo.draft_head(h, W, d2t, V).ids)
    res0, scores0, _ = vp.head_fused(g, gamma, 1e-6, W, d2t, 5)
    assert np.array_equal(scores0, res0.logp)
