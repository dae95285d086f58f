"""Parity of the compressed draft head (FP8 E4M3 with row scales, MXFP4 with block exponents)
with its CPU oracle on the same seeded inputs: the quantised subset (codes, scales, d2t) bit for
bit, the step's ids under the near-tie rule and its logits / log-probs within the same bounds as
the bf16 head (both sides take exact products of the hidden state with the same code values; they
differ in summation order and in one rounding of the scale)."""
import numpy as np
import pytest
import torch

import paper_2603_05210_amd as vt
from oracle import vq_oracle as vq
from paper_2603_05210_amd import synth
from tests.parity_util import check_head, to_dev_bf16

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
FMTS = [vq.FMT_FP8, vq.FMT_MXFP4]
assert (vt.VT_Q_FP8_E4M3, vt.VT_Q_MXFP4) == (vq.FMT_FP8, vq.FMT_MXFP4)


def _say(msg):
    print(msg, flush=True)


def build_both(W_u16, ids, fmt, W_dev=None):
    W_dev = to_dev_bf16(W_u16) if W_dev is None else W_dev
    codes, scales, d2t = vt.vt_build_subset_q(W_dev, torch.from_numpy(ids).to(DEV), fmt)
    torch.cuda.synchronize()
    o_codes, o_scales, o_d2t = vq.build_subset_q(W_u16, ids, fmt)
    assert np.array_equal(d2t.cpu().numpy(), o_d2t)
    g_scales = scales.cpu().numpy()
    assert np.array_equal(g_scales.view(np.uint32) if fmt == vq.FMT_FP8 else g_scales, o_scales.view(np.uint32) if fmt == vq.FMT_FP8 else o_scales), "scales differ"
    slab = 16384
    for a in range(0, len(ids), slab):
        assert np.array_equal(codes[a:a + slab].cpu().numpy(), o_codes[a:a + slab]), "codes differ in rows %d.." % a
    return codes, scales, d2t, o_codes, o_scales, o_d2t


def run_gpu(h_u16, codes, scales, fmt, d2t, k):
    Vd = codes.shape[0]
    logits = torch.full((1, Vd), float("nan"), dtype=torch.float32, device=DEV)
    lse = torch.full((1,), float("nan"), dtype=torch.float32, device=DEV)
    ids, lp = vt.vt_draft_head_q(to_dev_bf16(h_u16), codes, scales, fmt, d2t, k, logits_out=logits, lse_out=lse)
    torch.cuda.synchronize()
    ids2, lp2 = vt.vt_draft_head_q(to_dev_bf16(h_u16), codes, scales, fmt, d2t, k)   # the timed entry gives the same
    torch.cuda.synchronize()
    assert torch.equal(ids, ids2) and torch.equal(lp, lp2)
    return ids.cpu().numpy(), lp.cpu().numpy(), logits.cpu().numpy(), lse.cpu().numpy()


CASES = [
    # H, V, Vd, k
    (2048, 300, 77, 1),
    (2048, 40, 5, 5),          # k == V_draft, fewer rows than waves
    (4096, 6000, 4099, 10),
    (2048, 9000, 4380, 16),
    (4096, 3000, 1, 1),        # one draft token
    (2048, 40000, 33001, 7),
    (4096, 14000, 13264, 10),  # the paper's general-purpose size (Section 2.6)
]


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("H,V,Vd,k", CASES + [(1024, 5000, 2500, 3)])
def test_compressed_head_small_cases(fmt, H, V, Vd, k):
    if fmt == vq.FMT_MXFP4 and H == 1024:
        pytest.skip("MXFP4 step serves H = 2048 and 4096")
    _say("q case fmt=%d H=%d V=%d Vd=%d k=%d" % (fmt, H, V, Vd, k))
    seed = H + Vd + k
    W = synth.gen_W(seed, V, H, std=0.05)
    W[V // 2] = 0                                   # an all-zero row
    W[V // 3, 32:96] = 0                            # all-zero blocks
    h = synth.gen_h(seed, 1, H)
    ids = synth.zipf_subset(seed, V, Vd)
    codes, scales, d2t, o_codes, o_scales, o_d2t = build_both(W, ids, fmt)
    g_ids, g_lp, g_z, g_lse = run_gpu(h, codes, scales, fmt, d2t, k)
    ora = vq.draft_head_q(h, o_codes, o_scales, fmt, o_d2t, k)
    _say("  %s" % check_head(g_ids, g_lp, ora, o_d2t, gpu_logits=g_z, gpu_lse=g_lse))


@pytest.mark.parametrize("fmt", FMTS)
def test_compressed_head_ties_and_zero_hidden_state(fmt):
    """Duplicate rows give bit-equal logits: the lower draft index must come first; h = 0 gives
    the uniform distribution and the first k draft tokens."""
    H, V, k = 2048, 3000, 8
    W = synth.gen_W(21, V, H, std=0.05)
    for dst in (5, 900, 2100, 2999):
        W[dst] = W[1500]
    ids = np.arange(V, dtype=np.int32)
    codes, scales, d2t, o_codes, o_scales, o_d2t = build_both(W, ids, fmt)
    h = synth.bf16_to_f32(W[1500]) * 40.0          # points at the duplicated row
    h = synth.f32_to_bf16(h).reshape(1, H)
    g_ids, g_lp, g_z, _ = run_gpu(h, codes, scales, fmt, d2t, k)
    ora = vq.draft_head_q(h, o_codes, o_scales, fmt, o_d2t, k)
    assert list(g_ids[0][:5]) == [5, 900, 1500, 2100, 2999] == list(ora.ids[0][:5])
    z0 = run_gpu(np.zeros((1, H), dtype=np.uint16), codes, scales, fmt, d2t, k)
    assert np.all(z0[2] == 0.0) and list(z0[0][0]) == list(range(k)) and np.allclose(z0[1], -np.log(V), atol=1e-5)


def test_compressed_head_argument_errors():
    L = vt.lib()
    F = 0x1000
    wsb = vt.vt_draft_head_q_workspace_bytes(1, 1, 4096, 4096, 10)
    assert wsb > 0
    assert vt.vt_draft_head_q_workspace_bytes(1, 2, 4096, 4096, 10) == 0       # one row only
    assert vt.vt_draft_head_q_workspace_bytes(2, 1, 1024, 4096, 10) == 0       # MXFP4: H 2048 or 4096
    assert vt.vt_draft_head_q_workspace_bytes(3, 1, 4096, 4096, 10) == 0       # unknown format
    assert L.vt_draft_head_q(F, 2, 4096, F, F, 1, F, 4096, 10, F, F, F, wsb, None) == 2
    assert L.vt_draft_head_q(F, 1, 4096, F, F, 1, F, 4096, 17, F, F, F, wsb, None) == 3
    assert L.vt_draft_head_q(F, 1, 4096, F, F, 1, F, 4096, 10, F, F, F, wsb - 1, None) == 6
    assert L.vt_draft_head_q(None, 1, 4096, F, F, 1, F, 4096, 10, F, F, F, wsb, None) == 1
    assert L.vt_draft_head_q(F, 1, 4096, F + 4, F, 1, F, 4096, 10, F, F, F, wsb, None) == 7
    assert L.vt_build_subset_q(F, 1000, 4096, F, 10, 7, F, F, F, None) == 2
    assert L.vt_build_subset_q(F, 1000, 4096, F, 10, 1, None, F, F, None) == 1
    assert L.vt_subset_q_code_bytes(1, 1000, 4096) == 1000 * 4096 and L.vt_subset_q_scale_bytes(1, 1000, 4096) == 4000
    assert L.vt_subset_q_code_bytes(2, 1000, 4096) == 1000 * 2048 and L.vt_subset_q_scale_bytes(2, 1000, 4096) == 1000 * 128
    assert L.vt_subset_q_code_bytes(2, 1000, 4112) == 0


# ------------------------------------------------------------------ full-size workloads
@pytest.fixture(scope="module")
def W4096():
    _say("generating W[128256,4096]")
    W = synth.gen_W(0, synth.FULL_VOCAB, 4096)
    return W, to_dev_bf16(W)


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("Vd", [4096, 13264, 32768, 128256])
def test_compressed_vocab_sweep_full_size(W4096, fmt, Vd):
    """The metric's curve (one row, H = 4096, V_draft up to the full vocabulary) over the compressed
    forms: the whole quantised subset and every logit against the oracle."""
    W, W_dev = W4096
    ids = synth.zipf_subset(0, synth.FULL_VOCAB, Vd)
    codes, scales, d2t, o_codes, o_scales, o_d2t = build_both(W, ids, fmt, W_dev=W_dev)
    h = synth.gen_h(0, 1, 4096)
    g_ids, g_lp, g_z, g_lse = run_gpu(h, codes, scales, fmt, d2t, 10)
    ora = vq.draft_head_q(h, o_codes, o_scales, fmt, o_d2t, 10)
    _say("q fmt=%d Vd=%d %s" % (fmt, Vd, check_head(g_ids, g_lp, ora, o_d2t, gpu_logits=g_z, gpu_lse=g_lse)))
