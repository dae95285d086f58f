"""Parity of the head's fused neighbours (feature-fusion projection, RMSNorm on the way into the
head, path scores on the way out) with their CPU oracle.  bf16 outputs (the projection, the
normalised state) are compared as bit patterns: equal, or one unit in the last place apart where
the fp32 value both sides round sits on a rounding boundary (the two sides add in different
orders), and that on a small share of the elements only."""
import numpy as np
import pytest
import torch

import paper_2603_05210_amd as vt
from oracle import vp_oracle as vp
from oracle import vt_oracle as vo
from paper_2603_05210_amd import synth
from tests.parity_util import ABS_TOL, check_head, dev_bits, to_dev_bf16

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _say(msg):
    print(msg, flush=True)


def assert_bf16_close(got_u16, want_u16, what, max_share=0.02, abs_slack=2e-5):
    g = synth.bf16_to_f32(got_u16).astype(np.float64)
    w = synth.bf16_to_f32(want_u16).astype(np.float64)
    differs = got_u16 != want_u16
    # one bf16 unit in the last place of the larger magnitude (8 significant bits); results that
    # cancel to almost nothing carry the fp32 sums' own absolute error (orders differ), many units
    # of so small a value: abs_slack covers that
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.maximum(np.abs(g), np.abs(w)), 1e-30))) - 7)
    assert np.all(np.abs(g - w) <= ulp * 1.0001 + abs_slack), what
    assert differs.mean() <= max_share, (what, differs.mean())
    return float(differs.mean())


@pytest.mark.parametrize("rows,d_in,d_out", [
    (1, 192, 64), (1, 3072, 1024), (2, 1536, 520), (3, 200, 77), (4, 12288, 300),
    (5, 192, 64), (16, 1544, 260), (40, 3072, 1024), (130, 264, 129), (300, 1536, 512),
])
def test_feature_fusion_small_cases(rows, d_in, d_out):
    _say("fusion rows=%d d_in=%d d_out=%d" % (rows, d_in, d_out))
    x = synth.gen_h(rows + d_out, rows, d_in)
    W = synth.gen_W(rows + d_in, d_out, d_in, std=0.03)
    g = vt.vt_feature_fusion(to_dev_bf16(x), to_dev_bf16(W))
    torch.cuda.synchronize()
    share = assert_bf16_close(dev_bits(g), vp.feature_fusion(x, W), "fusion output")
    _say("  differing elements: %.4f" % share)


@pytest.mark.parametrize("rows", [1, 4, 9, 200])
def test_feature_fusion_exact_arithmetic_is_bit_exact(rows):
    d_in, d_out = 768, 260
    x = synth.small_int_bf16(3, 0, (rows, d_in))
    W = synth.small_int_bf16(3, 1, (d_out, d_in))
    g = vt.vt_feature_fusion(to_dev_bf16(x), to_dev_bf16(W))
    torch.cuda.synchronize()
    want = vp.feature_fusion(x, W)
    got = dev_bits(g)
    # small-integer sums are exact in fp32 in any order; the one rounding to bf16 is the same on both sides
    assert np.array_equal(got, want)


@pytest.mark.parametrize("rows", [1, 64])
def test_feature_fusion_full_size(rows):
    """Table 1's layer: d = 4096, three concatenated features."""
    d = 4096
    x = synth.gen_h(5, rows, 3 * d)
    W = synth.gen_W(5, d, 3 * d)
    g = vt.vt_feature_fusion(to_dev_bf16(x), to_dev_bf16(W))
    torch.cuda.synchronize()
    share = assert_bf16_close(dev_bits(g), vp.feature_fusion(x, W), "fusion output, full size")
    _say("fusion full size rows=%d: differing elements %.4f" % (rows, share))


FUSED = [
    # rows, H, V, Vd, k
    (1, 4096, 6000, 4099, 10),     # normalised inside the one-row kernel
    (1, 2048, 300, 77, 1),
    (1, 512, 3000, 1500, 16),
    (1, 4096, 14000, 13264, 10),
    (1, 264, 2000, 1500, 3),       # one row through the generic streaming kernel
    (2, 1024, 9000, 4099, 5),
    (8, 2048, 12000, 9001, 16),      # the kernel for a few rows behind the separate norm kernel
    (10, 4096, 20000, 13264, 8),
    (24, 4096, 6000, 4099, 10),      # two groups of rows
    (16, 4096, 300, 100, 3),         # fewer W_sub rows per workgroup than waves
    (40, 512, 2000, 700, 8),
    (300, 1024, 3000, 1300, 10),
]


@pytest.mark.parametrize("rows,H,V,Vd,k", FUSED)
def test_fused_norm_head_scores(rows, H, V, Vd, k):
    _say("fused rows=%d H=%d V=%d Vd=%d k=%d" % (rows, H, V, Vd, k))
    seed = rows * 7 + H + k
    W = synth.gen_W(seed, V, H, std=0.05)
    ids = synth.zipf_subset(seed, V, Vd)
    g = synth.f32_to_bf16(synth.bf16_to_f32(synth.gen_h(seed, rows, H, peaked_frac=0.2 if rows > 4 else 0.0)) * 3.7)
    gamma = synth.f32_to_bf16((1.0 + 0.2 * synth.normal(seed, 9, 0, H)).astype(np.float32))
    parent = (-np.abs(synth.normal(seed, 10, 0, rows)) * 2.0).astype(np.float32)
    eps = 1e-5
    W_sub, d2t = vt.vt_build_subset(to_dev_bf16(W), torch.from_numpy(ids).to(DEV))
    logits = torch.full((rows, Vd), float("nan"), dtype=torch.float32, device=DEV)
    lse = torch.full((rows,), float("nan"), dtype=torch.float32, device=DEV)
    h_out = torch.zeros((rows, H), dtype=torch.int16, device=DEV).view(torch.bfloat16)
    g_ids, g_sc = vt.vt_draft_head_fused(to_dev_bf16(g), to_dev_bf16(gamma), eps, W_sub, d2t, k,
                                         parent_scores=torch.from_numpy(parent).to(DEV), logits_out=logits, lse_out=lse, h_out=h_out)
    torch.cuda.synchronize()
    n_ids, n_sc = vt.vt_draft_head_fused(to_dev_bf16(g), to_dev_bf16(gamma), eps, W_sub, d2t, k,
                                         parent_scores=torch.from_numpy(parent).to(DEV))
    torch.cuda.synchronize()
    assert torch.equal(g_ids, n_ids) and torch.equal(g_sc, n_sc)        # the timed entry gives the same
    res, scores, h = vp.head_fused(g, gamma, eps, W[ids], ids, k, parent)
    share = assert_bf16_close(dev_bits(h_out), h, "normalised state", max_share=0.01)
    # the head itself, on the state the GPU normalised (so that every logit can be compared tightly)
    ora = vo.draft_head(dev_bits(h_out), W[ids], ids, k)
    g_lp = (g_sc.cpu().numpy().astype(np.float64) - parent[:, None].astype(np.float64)).astype(np.float32)
    st = check_head(g_ids.cpu().numpy(), g_lp, ora, ids, gpu_logits=logits.cpu().numpy(), gpu_lse=lse.cpu().numpy())
    _say("  h differing %.4f; %s" % (share, st))
    # and the whole chain against the oracle's own chain: scores of the tokens both sides report
    want = {(r, int(t)): float(s) for r in range(rows) for t, s in zip(res.ids[r], scores[r])}
    for r in range(rows):
        for t, s in zip(g_ids.cpu().numpy()[r], g_sc.cpu().numpy()[r]):
            if (r, int(t)) in want:
                assert abs(want[(r, int(t))] - float(s)) <= ABS_TOL
    # without parents the scores are the log-probabilities
    p_ids, p_sc = vt.vt_draft_head_fused(to_dev_bf16(g), to_dev_bf16(gamma), eps, W_sub, d2t, k)
    torch.cuda.synchronize()
    assert np.array_equal(p_ids.cpu().numpy(), g_ids.cpu().numpy())
    assert np.max(np.abs(p_sc.cpu().numpy() - g_lp)) <= 1e-5


def test_whole_draft_step_chain_fusion_to_scores():
    """x -> feature fusion -> RMSNorm -> trimmed head -> path scores, all on the GPU, against the oracle's chain."""
    d, V, Vd, k, rows = 1024, 9000, 4380, 8, 1
    x = synth.gen_h(71, rows, 3 * d)
    Wfc = synth.gen_W(71, d, 3 * d, std=0.02)
    W = synth.gen_W(72, V, d, std=0.05)
    ids = synth.zipf_subset(72, V, Vd)
    gamma = synth.f32_to_bf16(np.ones(d, dtype=np.float32))
    parent = np.array([-1.25], dtype=np.float32)
    W_sub, d2t = vt.vt_build_subset(to_dev_bf16(W), torch.from_numpy(ids).to(DEV))
    g_dev = vt.vt_feature_fusion(to_dev_bf16(x), to_dev_bf16(Wfc))
    g_ids, g_sc = vt.vt_draft_head_fused(g_dev, to_dev_bf16(gamma), 1e-6, W_sub, d2t, k, parent_scores=torch.from_numpy(parent).to(DEV))
    torch.cuda.synchronize()
    res, scores, _ = vp.head_fused(vp.feature_fusion(x, Wfc), gamma, 1e-6, W[ids], ids, k, parent)
    t2d = {int(t): j for j, t in enumerate(ids)}
    for p in range(k):
        gt, ot = int(g_ids[0, p]), int(res.ids[0, p])
        if gt != ot:
            assert abs(float(res.z[0, t2d[gt]]) - float(res.z[0, t2d[ot]])) <= ABS_TOL
        assert abs(float(g_sc[0, p]) - (float(res.z[0, t2d[gt]]) - float(res.lse[0]) + float(parent[0]))) <= ABS_TOL


def test_fusion_and_fused_head_argument_errors():
    L = vt.lib()
    F = 0x1000
    assert L.vt_feature_fusion(None, 1, 192, F, 64, F, None) == 1
    assert L.vt_feature_fusion(F, 0, 192, F, 64, F, None) == 2
    assert L.vt_feature_fusion(F, 1, 196, F, 64, F, None) == 2
    assert L.vt_feature_fusion(F + 8, 1, 192, F, 64, F, None) == 7
    need = vt.vt_draft_head_fused_workspace_bytes(8, 2048, 9000, 10)
    assert need >= vt.vt_draft_head_workspace_bytes(8, 2048, 9000, 10) + 8 * 2048 * 2
    import ctypes
    e = ctypes.c_float(1e-5)
    assert L.vt_draft_head_fused(F, None, e, None, 8, 2048, F, F, 9000, 10, F, F, F, need, None) == 1
    assert L.vt_draft_head_fused(F, F, e, None, 8, 2048, F, F, 9000, 10, F, F, F, need - 256, None) == 6
    assert L.vt_draft_head_fused(F, F, ctypes.c_float(-1.0), None, 8, 2048, F, F, 9000, 10, F, F, F, need, None) == 2
    assert L.vt_draft_head_fused(F, F, e, None, 8, 2048, F, F, 9000, 0, F, F, F, need, None) == 3
