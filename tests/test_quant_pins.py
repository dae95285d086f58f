"""Pins of the compressed-head oracle (oracle/vq_oracle.py) to facts outside itself: the two
formats' value tables as their specifications give them, a library's own E4M3 conversion,
exhaustive nearest-value search in exact rational arithmetic, round trips of representable
values, the formats' error bounds on Gaussian rows, and the head's invariants."""
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import vq_oracle as vq
from oracle import vt_oracle as vo
from paper_2603_05210_amd import synth


# ---------------------------------------------------------------- E4M3
def test_e4m3_table_is_the_ocp_format():
    t = vq.e4m3_table()
    assert t[0x00] == 0.0 and t[0x38] == 1.0 and t[0x7E] == 448.0 and t[0x01] == 2.0 ** -9 and t[0x08] == 2.0 ** -6
    assert t[0x3C] == 1.5 and t[0xB8] == -1.0 and t[0xFE] == -448.0
    assert np.isnan(t[0x7F]) and np.isnan(t[0xFF]) and np.isfinite(t).sum() == 254
    pos = t[:0x7F]
    assert np.all(np.diff(pos) > 0)                       # codes order the magnitudes
    # the library's decode of every finite code
    lib = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float32).numpy()
    fin = np.isfinite(t)
    assert np.array_equal(lib[fin], t[fin])


def test_e4m3_encode_matches_the_library_conversion_and_brute_force():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.normal(0, 100, 20000), rng.normal(0, 1, 20000), rng.normal(0, 0.01, 20000),
                        rng.uniform(-460, 460, 20000), [0.0, -0.0, 448.0, -448.0, 2.0 ** -9, 2.0 ** -10, 3 * 2.0 ** -10,
                                                         463.9, 0.0175, 2.0 ** -6, 2.0 ** -6 - 2.0 ** -11]]).astype(np.float32)
    # every midpoint between neighbouring codes (the ties) and a hair to each side
    t = vq.e4m3_table()[:0x7F].astype(np.float64)
    mid = ((t[:-1] + t[1:]) / 2).astype(np.float32)
    x = np.concatenate([x, mid, -mid, np.nextafter(mid, np.float32(0)), np.nextafter(mid, np.float32(1e9))]).astype(np.float32)
    got = vq.e4m3_encode(x)
    lib = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    same_zero = (got & 0x7F) == 0
    assert np.array_equal(got[~same_zero], lib[~same_zero])
    assert np.all((lib[same_zero] & 0x7F) == 0)
    # brute force on a sample: the code whose value is nearest in exact arithmetic, even mantissa on ties
    table = [Fraction(float(v)) for v in vq.e4m3_table()[:0x7F]]
    for v in x[::97]:
        a = Fraction(abs(float(v)))
        best = min(range(0x7F), key=lambda c: (abs(table[c] - a), c & 1))
        assert (int(vq.e4m3_encode(np.array([v], dtype=np.float32))[0]) & 0x7F) == best, float(v)
    # saturation beyond the largest finite value
    assert list(vq.e4m3_encode(np.array([1000.0, -1e6, 464.0], dtype=np.float32))) == [0x7E, 0xFE, 0x7E]


def test_fp8_round_trip_scale_and_error_bound():
    W = synth.gen_W(3, 300, 512)
    W[7] = 0                                               # an all-zero row
    codes, scales = vq.quantize_fp8(W)
    w = synth.bf16_to_f32(W)
    amax = np.abs(w).max(axis=1)
    assert scales[7] == 1.0 and np.all(codes[7] == 0)
    ok = amax > 0
    assert np.allclose(scales[ok] * 448.0, amax[ok], rtol=1e-6)
    assert not np.any((codes & 0x7F) == 0x7F)
    # the row maximum maps to +-448
    assert np.all(np.max(codes[ok] & 0x7F, axis=1) == 0x7E)
    # error bound of the format: half a unit in the last place, 2^-4 relative for normal numbers
    # (3 mantissa bits), 2^-10 absolute below 2^-6, in units of the scale
    dq = vq.dequantize_fp8(codes, scales)
    x = np.abs(w / scales[:, None])
    bound = np.where(x >= 2.0 ** -6, x * 2.0 ** -4, 2.0 ** -10) * scales[:, None] * (1 + 1e-5)
    assert np.all(np.abs(dq - w) <= bound)
    # codes are a fixed point: quantising the dequantised values with the same scale returns them
    again = vq.e4m3_encode((dq / scales[:, None]).astype(np.float32))
    nz = (codes & 0x7F) != 0
    assert np.array_equal(again[nz], codes[nz])


# ---------------------------------------------------------------- MXFP4
def test_e2m1_values_and_exhaustive_nearest_value_rule():
    assert [vq.e2m1_value(n) for n in range(8)] == [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]
    assert [vq.e2m1_value(n) for n in range(8, 16)] == [-0.0, -0.5, -1.0, -1.5, -2.0, -3.0, -4.0, -6.0]
    grid = [Fraction(v) for v in (0, 0.5, 1, 1.5, 2, 3, 4, 6)]
    xs = [Fraction(n, 64) for n in range(0, 64 * 9)]       # every 1/64 up to 9: all midpoints included
    got = vq.e2m1_encode(np.array([float(v) for v in xs]))
    for v, g in zip(xs, got):
        want = min(range(8), key=lambda c: (abs(grid[c] - v), c & 1))
        assert int(g) == want, float(v)
    assert list(vq.e2m1_encode(np.array([-0.75, -6.5, -100.0, 5.0, 7.0]))) == [0xA, 0xF, 0xF, 0x6, 0x7]


def test_mxfp4_block_scale_packing_and_error_bound():
    H = 256
    W = synth.gen_W(5, 200, H, std=0.05)
    W[3, 32:64] = 0                                         # an all-zero block
    packed, eb = vq.quantize_mxfp4(W)
    assert packed.shape == (200, H // 2) and eb.shape == (200, H // 32) and eb[3, 1] == 127
    w = synth.bf16_to_f32(W).astype(np.float64).reshape(200, H // 32, 32)
    amax = np.abs(w).max(axis=2)
    scale = np.ldexp(1.0, eb.astype(np.int64) - 127)
    nzb = amax > 0
    # the shared exponent is floor(log2(amax)) - 2: the block maximum lands in [4, 8) scale units
    r = amax[nzb] / scale[nzb]
    assert np.all((r >= 4.0) & (r < 8.0))
    # packing: even element in the low nibble
    nib_lo, nib_hi = packed & 0xF, packed >> 4
    x = (w / scale[:, :, None]).reshape(200, H)
    assert np.array_equal(nib_lo, vq.e2m1_encode(x[:, 0::2])) and np.array_equal(nib_hi, vq.e2m1_encode(x[:, 1::2]))
    # error bound of the format in scale units: half a step (0.25 below 2, 0.5 below 4, 1 up to 6), and up to 2
    # where the block maximum saturates (values in (6, 8))
    dq = vq.dequantize_mxfp4(packed, eb).astype(np.float64)
    ax = np.abs(x)
    bound = np.select([ax <= 2, ax <= 4, ax <= 6], [0.25, 0.5, 1.0], default=2.0)
    err = np.abs(dq - synth.bf16_to_f32(W).astype(np.float64)).reshape(200, H // 32, 32) / scale[:, :, None]
    assert np.all(err.reshape(200, H) <= bound + 1e-12)
    # round trip: representable values with a power-of-two maximum come back exactly
    vals = np.array([0, 0.5, 1, 1.5, 2, 3, 4, 6, -0.5, -1, -1.5, -2, -3, -4, -6, 4] * 2, dtype=np.float32) * np.float32(2.0 ** -5)
    Wr = synth.f32_to_bf16(vals).reshape(1, 32)
    p2, e2 = vq.quantize_mxfp4(Wr)
    assert e2[0, 0] == 127 - 5 and np.array_equal(vq.dequantize_mxfp4(p2, e2)[0], vals)


# ---------------------------------------------------------------- subset and head
@pytest.mark.parametrize("fmt", [vq.FMT_FP8, vq.FMT_MXFP4])
def test_compressed_subset_is_the_compressed_matrix_restricted(fmt):
    V, H, Vd = 700, 128, 200
    W = synth.gen_W(8, V, H)
    ids = synth.zipf_subset(8, V, Vd)
    codes, scales, d2t = vq.build_subset_q(W, ids, fmt)
    full_codes, full_scales = vq.quantize(W, fmt)
    assert np.array_equal(codes, full_codes[ids]) and np.array_equal(scales, full_scales[ids]) and np.array_equal(d2t, ids)
    ident = np.arange(V, dtype=np.int32)
    c2, s2, d2 = vq.build_subset_q(W, ident, fmt)
    assert np.array_equal(c2, full_codes) and np.array_equal(d2, ident)


@pytest.mark.parametrize("fmt", [vq.FMT_FP8, vq.FMT_MXFP4])
def test_compressed_head_invariants(fmt):
    V, H, Vd, k = 900, 256, 333, 7
    W = synth.gen_W(9, V, H, std=0.05)
    h = synth.gen_h(9, 3, H)
    ids = synth.zipf_subset(9, V, Vd)
    codes, scales, d2t = vq.build_subset_q(W, ids, fmt)
    res = vq.draft_head_q(h, codes, scales, fmt, d2t, k)
    # logits are the plain product of the hidden state with the dequantised weights (library matmul in double)
    dq = vq.dequantize(codes, scales, fmt).astype(np.float64)
    z64 = synth.bf16_to_f32(h).astype(np.float64) @ dq.T
    assert np.max(np.abs(res.z - z64)) < 1e-4
    # restriction: the trimmed compressed head equals the full compressed head on V_d's rows, bit for bit
    fc, fs = vq.quantize(W, fmt)
    full = vq.draft_head_q(h, fc, fs, fmt, np.arange(V, dtype=np.int32), k)
    assert np.array_equal(res.z.view(np.uint32), full.z[:, ids].view(np.uint32))
    # normalisation over V_d, ordering, remap
    p = np.exp(res.z.astype(np.float64) - res.lse[:, None].astype(np.float64))
    assert np.allclose(p.sum(axis=1), 1.0, atol=1e-5)
    for r in range(3):
        order = sorted(range(Vd), key=lambda j: (-res.z[r, j], j))[:k]
        assert list(res.draft_idx[r]) == order and list(res.ids[r]) == [int(d2t[j]) for j in order]
    # rows are independent: a batch gives what its rows give one at a time, in any order, bit for bit
    for r in (2, 0):
        one = vq.draft_head_q(h[r:r + 1], codes, scales, fmt, d2t, k)
        assert np.array_equal(one.z.view(np.uint32), res.z[r:r + 1].view(np.uint32)) and np.array_equal(one.ids, res.ids[r:r + 1])
        assert np.array_equal(one.logp.view(np.uint32), res.logp[r:r + 1].view(np.uint32))
    # zero hidden state: uniform distribution, first k draft tokens
    z0 = vq.draft_head_q(np.zeros((1, H), dtype=np.uint16), codes, scales, fmt, d2t, k)
    assert np.allclose(z0.logp, -np.log(Vd), atol=1e-6) and list(z0.ids[0]) == list(d2t[:k])
    # compression error against the bf16 head stays within the formats' budget for these inputs
    zb = vo.logits(h, W[ids])
    rel = np.sqrt(np.mean((res.z - zb) ** 2) / np.mean(zb ** 2))
    assert rel < (0.04 if fmt == vq.FMT_FP8 else 0.2), rel
