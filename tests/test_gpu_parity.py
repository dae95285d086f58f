"""Parity of the HIP path (through the C ABI) with the CPU oracle on the same seeded inputs.

Small cases are compared in full (every logit, every id, every log-prob) at sizes that span
several tiles / waves / workgroups with ragged tails; the five full-size workloads are compared
in full too: every row's ids and log-probs, every row of the gathered W_sub, and every logit of
the one-row workloads and of a 256-row block of the tree-drafting ones.
"""
import numpy as np
import pytest
import torch

import paper_2603_05210_amd as vt
from oracle import vt_oracle as vo
from paper_2603_05210_amd import synth
from tests.parity_util import check_head, dev_bits, to_dev_bf16

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _say(msg):
    print(msg, flush=True)


def run_gpu(h_u16, Wsub_dev, d2t_dev, k, debug=True):
    h_dev = to_dev_bf16(h_u16)
    R = h_u16.shape[0]
    Vd = Wsub_dev.shape[0]
    logits = torch.full((R, Vd), float("nan"), dtype=torch.float32, device=DEV) if debug else None
    lse = torch.full((R,), float("nan"), dtype=torch.float32, device=DEV) if debug else None
    ids, lp = vt.vt_draft_head(h_dev, Wsub_dev, d2t_dev, k, logits_out=logits, lse_out=lse)
    torch.cuda.synchronize()
    return (ids.cpu().numpy(), lp.cpu().numpy(), None if logits is None else logits.cpu().numpy(),
            None if lse is None else lse.cpu().numpy())


def build_both(W_u16, ids_np):
    W_dev = to_dev_bf16(W_u16)
    ids_dev = torch.from_numpy(ids_np).to(DEV)
    Wsub_dev, d2t_dev = vt.vt_build_subset(W_dev, ids_dev)
    torch.cuda.synchronize()
    Wsub_o, d2t_o = vo.build_subset(W_u16, ids_np)
    assert np.array_equal(dev_bits(Wsub_dev), Wsub_o), "gather is not bit-exact"
    assert np.array_equal(d2t_dev.cpu().numpy(), d2t_o), "d2t differs"
    return Wsub_dev, d2t_dev, Wsub_o, d2t_o


SMALL = [
    # rows, H, V, Vd, k           streaming regime
    (1, 64, 300, 77, 1),
    (1, 2048, 6000, 4096, 1),
    (2, 520, 3000, 1001, 5),
    (3, 1024, 9000, 4099, 10),
    (4, 2048, 7000, 5003, 10),
    (7, 264, 2000, 1500, 3),
    (8, 2048, 12000, 9001, 16),
    (13, 512, 3000, 2049, 33),
    (16, 1024, 2000, 777, 64),
    (1, 4096, 40000, 33001, 10),
    # MFMA regime
    (17, 256, 1000, 300, 8),
    (33, 64, 500, 129, 1),
    (130, 512, 2000, 700, 16),
    (200, 1096, 3000, 1000, 8),
    (260, 264, 2000, 520, 33),
    (300, 1024, 3000, 1300, 64),
    (512, 512, 2000, 1030, 8),
]


EDGE = [
    # rows, H, V, Vd, k           degenerate and limit shapes
    (1, 8, 10, 1, 1),             # one draft token, minimum H
    (1, 8, 40, 5, 5),             # k == V_draft
    (20, 8, 40, 5, 5),            # the same through the MFMA regime
    (16, 72, 900, 600, 64),       # 16 rows, longest list, H not a multiple of 64
    (17, 72, 900, 600, 64),       # first row count of the MFMA regime, longest list, K tail
    (2, 64, 150000, 140000, 10),  # more workgroup partials than the fused merge takes
    (9, 128, 150000, 133000, 3),
    (2, 256, 70000, 65600, 4),    # wide vocabulary, fused merge
    (2, 256, 150000, 140000, 10),  # the same with more partials than the fused merge takes
    (5, 256, 70000, 66001, 10),   # matrix-core streaming kernel: ragged last 16-row group and workgroup
    (9, 256, 131000, 130000, 5),
    (16, 512, 70000, 69000, 16),
    (16, 4096, 70000, 65536, 8),  # hidden states leave no LDS for staging: direct-load form
    (16, 4096, 131200, 131072, 8),  # 16 rows x 512 W_sub rows per workgroup: LDS exactly full, goes to the GEMM regime
    (1, 16384, 3000, 2500, 10),   # a very wide hidden state, one row
    (16, 8192, 2000, 1500, 5),    # 16 rows whose hidden states do not fit LDS: matrix-core regime
    (2048, 64, 600, 500, 4),      # many rows, narrow everything
    (1, 2048, 130000, 128256, 64),  # longest list over the widest vocabulary
    (129, 64, 700, 257, 16),      # one row and one token past a tile edge
    (256, 128, 2000, 512, 16),    # exact tile multiples
]


@pytest.mark.parametrize("rows,H,V,Vd,k", SMALL + EDGE)
def test_small_cases_full_comparison(rows, H, V, Vd, k):
    _say("case rows=%d H=%d V=%d Vd=%d k=%d" % (rows, H, V, Vd, k))
    seed = rows * 1000 + k
    W = synth.gen_W(seed, V, H, std=0.05)
    h = synth.gen_h(seed, rows, H, peaked_frac=0.1 if rows >= 10 else 0.0)
    ids = synth.zipf_subset(seed, V, Vd)
    Wsub_dev, d2t_dev, Wsub_o, d2t_o = build_both(W, ids)
    g_ids, g_lp, g_z, g_lse = run_gpu(h, Wsub_dev, d2t_dev, k)
    ora = vo.draft_head(h, Wsub_o, d2t_o, k)
    st = check_head(g_ids, g_lp, ora, d2t_o, gpu_logits=g_z, gpu_lse=g_lse)
    _say("  %s" % st)
    # the timed entry point (no logits stored) gives the same answer as the test hook
    n_ids, n_lp, _, _ = run_gpu(h, Wsub_dev, d2t_dev, k, debug=False)
    assert np.array_equal(n_ids, g_ids) and np.array_equal(n_lp, g_lp)


@pytest.mark.parametrize("rows", [1, 5, 16, 40, 300])
def test_exact_arithmetic_cases_are_bit_exact(rows):
    """Small-integer inputs: every fp32 sum is exact in any order, ties abound, so logits, ids
    and their order must equal the oracle's bit for bit (stresses the tie rule across lanes,
    waves, tiles and workgroups)."""
    H, Vd, k = 512, 3001, 12
    _say("exact rows=%d" % rows)
    Wb = synth.small_int_bf16(5, 0, (Vd, H))
    hb = synth.small_int_bf16(5, 1, (rows, H))
    d2t = np.arange(Vd, dtype=np.int32)[::-1].copy()  # a non-trivial map
    W_dev = to_dev_bf16(Wb)
    d2t_dev = torch.from_numpy(d2t).to(DEV)
    g_ids, g_lp, g_z, g_lse = run_gpu(hb, W_dev, d2t_dev, k)
    ora = vo.draft_head(hb, Wb, d2t, k)
    assert np.array_equal(g_z.view(np.uint32), ora.z.view(np.uint32))
    assert np.array_equal(g_ids, ora.ids)
    assert np.max(np.abs(g_lp - ora.logp)) < 1e-3


@pytest.mark.parametrize("rows", [5, 11, 16])
def test_exact_arithmetic_matrix_core_streaming(rows):
    """The same through the matrix-core streaming kernel (several rows, H % 256 == 0, a
    vocabulary wide enough for 16-row groups on every wave)."""
    H, Vd, k = 256, 66003, 12
    _say("exact (matrix-core streaming) rows=%d" % rows)
    assert vt.vt_draft_head_regime(rows, H, Vd, k) == 0
    Wb = synth.small_int_bf16(6, 0, (Vd, H))
    hb = synth.small_int_bf16(6, 1, (rows, H))
    d2t = np.arange(Vd, dtype=np.int32)[::-1].copy()
    g_ids, g_lp, g_z, g_lse = run_gpu(hb, to_dev_bf16(Wb), torch.from_numpy(d2t).to(DEV), k)
    ora = vo.draft_head(hb, Wb, d2t, k)
    assert np.array_equal(g_z.view(np.uint32), ora.z.view(np.uint32))
    assert np.array_equal(g_ids, ora.ids)
    assert np.max(np.abs(g_lp - ora.logp)) < 1e-3


# The kernel for 2..16 rows at H = 2048 / 4096 (16 waves share every block of 16 W_sub rows; results
# travel workgroup -> group of 16 workgroups -> call): one workgroup, one group, a last group of one
# workgroup, ragged last blocks, every row-count set, k from 1 to 16.
FEW_ROWS = [
    (5, 4096, 500, 16, 16),      # a single workgroup with a single full block, k == V_draft
    (3, 2048, 300, 17, 5),       # two workgroups of 9 and 8 rows
    (2, 4096, 6000, 4096, 10),   # 256 workgroups of exactly one block
    (13, 4096, 3000, 257, 1),    # 17 workgroups: the second group has one member
    (10, 2048, 9000, 4380, 8),
    (8, 4096, 20000, 13264, 10),
    (16, 2048, 5000, 4097, 16),
    (16, 4096, 9000, 8200, 16),  # 32 or 33 rows per workgroup: a ragged third block
    (4, 2048, 70000, 66001, 10),
    # more than 16 rows: groups of 16 rows on workgroups of their own, side by side over the same W_sub rows
    (17, 4096, 6000, 4099, 10),   # a second group of one row
    (32, 4096, 3000, 2049, 8),    # two full groups; 128 runs of 16 or 17 rows
    (40, 2048, 9000, 4380, 16),   # three groups (80 runs)
    (64, 4096, 20000, 13264, 10),  # four groups
    (33, 2048, 300, 100, 3),      # fewer runs than a multiple of 8: the plain block numbering
]


@pytest.mark.parametrize("rows,H,V,Vd,k", FEW_ROWS)
def test_few_rows_kernel_full_comparison(rows, H, V, Vd, k):
    _say("few rows: rows=%d H=%d V=%d Vd=%d k=%d" % (rows, H, V, Vd, k))
    seed = rows * 977 + k
    W = synth.gen_W(seed, V, H, std=0.05)
    h = synth.gen_h(seed, rows, H, peaked_frac=0.1 if rows >= 10 else 0.0)
    ids = synth.zipf_subset(seed, V, Vd)
    Wsub_dev, d2t_dev, Wsub_o, d2t_o = build_both(W, ids)
    g_ids, g_lp, g_z, g_lse = run_gpu(h, Wsub_dev, d2t_dev, k)
    ora = vo.draft_head(h, Wsub_o, d2t_o, k)
    st = check_head(g_ids, g_lp, ora, d2t_o, gpu_logits=g_z, gpu_lse=g_lse)
    _say("  %s" % st)
    # the timed entry point, three times over one workspace (every counter must be back at zero)
    ws = vt.new_workspace(vt.vt_draft_head_workspace_bytes(rows, H, Vd, k), DEV)
    h_dev = to_dev_bf16(h)
    for _ in range(3):
        n_ids, n_lp = vt.vt_draft_head(h_dev, Wsub_dev, d2t_dev, k, workspace=ws)
        torch.cuda.synchronize()
        assert np.array_equal(n_ids.cpu().numpy(), g_ids) and np.array_equal(n_lp.cpu().numpy(), g_lp)


@pytest.mark.parametrize("rows,H", [(2, 4096), (7, 2048), (12, 4096), (16, 2048), (23, 4096), (64, 2048)])
def test_exact_arithmetic_few_rows_kernel(rows, H):
    """Small-integer inputs through the kernel for 2..16 rows: logits bit for bit, ties (many) by draft index."""
    Vd, k = 5001, 12
    _say("exact (few rows) rows=%d H=%d" % (rows, H))
    Wb = synth.small_int_bf16(7, 0, (Vd, H), lo=-2, hi=2)
    hb = synth.small_int_bf16(7, 1, (rows, H), lo=-2, hi=2)
    d2t = np.arange(Vd, dtype=np.int32)[::-1].copy()
    g_ids, g_lp, g_z, g_lse = run_gpu(hb, to_dev_bf16(Wb), torch.from_numpy(d2t).to(DEV), k)
    ora = vo.draft_head(hb, Wb, d2t, k)
    assert np.array_equal(g_z.view(np.uint32), ora.z.view(np.uint32))
    assert np.array_equal(g_ids, ora.ids)
    assert np.max(np.abs(g_lp - ora.logp)) < 1e-3


@pytest.mark.parametrize("rows", [1, 8, 64])
def test_one_hot_hidden_state_is_bit_exact(rows):
    H, Vd, k = 1024, 2500, 7
    W = synth.gen_W(9, Vd, H, std=0.05)
    h = np.zeros((rows, H), dtype=np.uint16)
    for r in range(rows):
        h[r, (r * 37 + 5) % H] = synth.f32_to_bf16(np.array([(-1.0) ** r * (0.5 + r)], dtype=np.float32))[0]
    d2t = np.arange(Vd, dtype=np.int32)
    g_ids, g_lp, g_z, _ = run_gpu(h, to_dev_bf16(W), torch.from_numpy(d2t).to(DEV), k)
    ora = vo.draft_head(h, W, d2t, k)
    assert np.array_equal(g_z.view(np.uint32), ora.z.view(np.uint32))
    assert np.array_equal(g_ids, ora.ids)


@pytest.mark.parametrize("rows", [1, 4, 100])
def test_zero_hidden_state(rows):
    H, Vd, k = 256, 1234, 9
    W = synth.gen_W(2, Vd, H)
    d2t = (np.arange(Vd, dtype=np.int32) * 3 + 1)
    h = np.zeros((rows, H), dtype=np.uint16)
    g_ids, g_lp, g_z, g_lse = run_gpu(h, to_dev_bf16(W), torch.from_numpy(d2t).to(DEV), k)
    assert np.all(g_z == 0.0)
    assert np.array_equal(g_ids, np.tile(d2t[:k], (rows, 1)))
    assert np.allclose(g_lp, -np.log(float(Vd)), atol=1e-5)


def test_identity_subset_and_unsorted_ids():
    V, H = 1500, 256
    W = synth.gen_W(4, V, H, std=0.05)
    W[100] = W[900]
    W[40] = W[900]
    h = synth.gen_h(4, 3, H)
    ident = np.arange(V, dtype=np.int32)
    Wsub_dev, d2t_dev, Wsub_o, d2t_o = build_both(W, ident)
    assert np.array_equal(dev_bits(Wsub_dev), W)
    g_ids, g_lp, g_z, _ = run_gpu(h, Wsub_dev, d2t_dev, 10)
    check_head(g_ids, g_lp, vo.draft_head(h, Wsub_o, d2t_o, 10), d2t_o, gpu_logits=g_z)
    # unsorted ids: the position in the list is the draft index and decides ties
    ids = np.array([900, 7, 100, 1499, 40, 0, 650], dtype=np.int32)
    Wsub_dev, d2t_dev, Wsub_o, d2t_o = build_both(W, ids)
    g_ids, g_lp, g_z, _ = run_gpu(h, Wsub_dev, d2t_dev, 7)
    ora = vo.draft_head(h, Wsub_o, d2t_o, 7)
    assert np.array_equal(g_ids, ora.ids)
    for r in range(3):
        pos = {int(t): p for p, t in enumerate(g_ids[r])}
        assert pos[900] < pos[100] < pos[40]


def test_build_subset_rejects_bad_ids_and_leaves_outputs_alone():
    V, H = 500, 64
    W_dev = to_dev_bf16(synth.gen_W(1, V, H))
    out_W = torch.full((3, H), 7, dtype=torch.int16, device=DEV).view(torch.bfloat16)
    out_d = torch.full((3,), -5, dtype=torch.int32, device=DEV)
    for bad, code in (([1, 2, 500], 4), ([1, -1, 2], 4), ([9, 2, 9], 5)):
        ids = torch.tensor(bad, dtype=torch.int32, device=DEV)
        with pytest.raises(vt.VtError) as e:
            vt.vt_build_subset(W_dev, ids, out_W, out_d)
        assert e.value.status == code
        torch.cuda.synchronize()
        assert torch.all(out_d == -5) and torch.all(out_W.view(torch.int16) == 7)


def test_results_do_not_depend_on_run(capsys):
    rows, H, Vd, k = 6, 1024, 20011, 10
    W = synth.gen_W(12, Vd, H)
    h = synth.gen_h(12, rows, H)
    W_dev, d2t_dev = to_dev_bf16(W), torch.arange(Vd, dtype=torch.int32, device=DEV)
    a = run_gpu(h, W_dev, d2t_dev, k)
    for _ in range(3):
        b = run_gpu(h, W_dev, d2t_dev, k)
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1].view(np.uint32), b[1].view(np.uint32))
        assert np.array_equal(a[2].view(np.uint32), b[2].view(np.uint32))


@pytest.mark.parametrize("rows,H,Vd,k", [(1, 1024, 30011, 10), (6, 512, 9001, 4), (300, 512, 3000, 8),
                                         (8, 4096, 9001, 8), (24, 2048, 5000, 10)])
def test_hip_graph_replays_match_eager(rows, H, Vd, k):
    """A captured draft step replays correctly (several replays, eager work in between): the
    step allocates nothing, takes no host round trip and its fused merge re-arms itself."""
    W = synth.gen_W(31, Vd, H, std=0.05)
    W_dev = to_dev_bf16(W)
    d2t_dev = torch.arange(Vd, dtype=torch.int32, device=DEV)
    hs = [to_dev_bf16(synth.gen_h(40 + i, rows, H)) for i in range(3)]
    h_in = hs[0].clone()
    ws = vt.new_workspace(vt.vt_draft_head_workspace_bytes(rows, H, Vd, k), DEV)
    ids = torch.empty((rows, k), dtype=torch.int32, device=DEV)
    lp = torch.empty((rows, k), dtype=torch.float32, device=DEV)
    eager = []
    for h in hs:
        a, b = vt.vt_draft_head(h, W_dev, d2t_dev, k)
        torch.cuda.synchronize()
        eager.append((a.cpu().numpy(), b.cpu().numpy()))
    vt.vt_draft_head(h_in, W_dev, d2t_dev, k, ids, lp, ws)  # warm: one-time kernel attributes are set
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        vt.vt_draft_head(h_in, W_dev, d2t_dev, k, ids, lp, ws)
    for rep in range(6):
        i = rep % 3
        h_in.copy_(hs[i])
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(ids.cpu().numpy(), eager[i][0]), "replay %d" % rep
        assert np.array_equal(lp.cpu().numpy().view(np.uint32), eager[i][1].view(np.uint32)), "replay %d" % rep
        junk = torch.randn(1000, device=DEV).sum().item()  # unrelated eager work between replays
        assert junk == junk


def test_calls_on_two_streams_do_not_disturb_each_other():
    """Single-launch (one- and two-row) steps interleaved on two streams, each with its own
    workspace and outputs: every call must give what it gives alone (the arrival counters of
    concurrent calls are distinct)."""
    H, Vd, k = 512, 20000, 10
    W_dev = to_dev_bf16(synth.gen_W(77, Vd, H, std=0.05))
    d2t_dev = torch.arange(Vd, dtype=torch.int32, device=DEV)
    hs = {r: to_dev_bf16(synth.gen_h(50 + r, r, H)) for r in (1, 2)}
    alone = {}
    for r, h in hs.items():
        a, b = vt.vt_draft_head(h, W_dev, d2t_dev, k)
        torch.cuda.synchronize()
        alone[r] = (a.cpu().numpy(), b.cpu().numpy())
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]   # default priority
    slots = []
    for si, st in enumerate(streams):
        for n in range(40):
            r = 1 + (n + si) % 2
            ws = vt.new_workspace(vt.vt_draft_head_workspace_bytes(r, H, Vd, k), DEV)
            ids = torch.empty((r, k), dtype=torch.int32, device=DEV)
            lp = torch.empty((r, k), dtype=torch.float32, device=DEV)
            slots.append((si, r, ws, ids, lp))
    torch.cuda.synchronize()
    for n in range(40):
        for si, st in enumerate(streams):
            _, r, ws, ids, lp = slots[si * 40 + n]
            with torch.cuda.stream(st):
                vt.vt_draft_head(hs[r], W_dev, d2t_dev, k, ids, lp, ws)
    torch.cuda.synchronize()
    for si, r, ws, ids, lp in slots:
        assert np.array_equal(ids.cpu().numpy(), alone[r][0])
        assert np.array_equal(lp.cpu().numpy().view(np.uint32), alone[r][1].view(np.uint32))


def test_few_row_calls_on_two_streams_do_not_disturb_each_other():
    """The same for the kernel that serves a few rows (8 rows and 20 rows: one and two groups of rows),
    whose arrival counters (groups of workgroups, groups of rows) also live in the call's own workspace."""
    H, Vd, k = 2048, 9000, 10
    W_dev = to_dev_bf16(synth.gen_W(79, Vd, H, std=0.05))
    d2t_dev = torch.arange(Vd, dtype=torch.int32, device=DEV)
    hs = {r: to_dev_bf16(synth.gen_h(70 + r, r, H)) for r in (8, 20)}
    alone = {}
    for r, h in hs.items():
        assert vt.vt_draft_head_regime(r, H, Vd, k) == 0
        a, b = vt.vt_draft_head(h, W_dev, d2t_dev, k)
        torch.cuda.synchronize()
        alone[r] = (a.cpu().numpy(), b.cpu().numpy())
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]   # default priority
    slots = []
    for si, st in enumerate(streams):
        for n in range(30):
            r = (8, 20)[(n + si) % 2]
            ws = vt.new_workspace(vt.vt_draft_head_workspace_bytes(r, H, Vd, k), DEV)
            ids = torch.empty((r, k), dtype=torch.int32, device=DEV)
            lp = torch.empty((r, k), dtype=torch.float32, device=DEV)
            slots.append((si, r, ws, ids, lp))
    torch.cuda.synchronize()
    for n in range(30):
        for si, st in enumerate(streams):
            _, r, ws, ids, lp = slots[si * 30 + n]
            with torch.cuda.stream(st):
                vt.vt_draft_head(hs[r], W_dev, d2t_dev, k, ids, lp, ws)
    torch.cuda.synchronize()
    for si, r, ws, ids, lp in slots:
        assert np.array_equal(ids.cpu().numpy(), alone[r][0])
        assert np.array_equal(lp.cpu().numpy().view(np.uint32), alone[r][1].view(np.uint32))


def test_graph_replays_while_many_eager_calls_run_on_another_stream():
    """A captured one-row step replays on one stream while more than a thousand eager one-row
    steps run on another: each call owns its arrival counter (in its workspace), so neither
    disturbs the other whatever the number of calls in flight."""
    H, Vd, k = 512, 20000, 10
    W_dev = to_dev_bf16(synth.gen_W(78, Vd, H, std=0.05))
    d2t_dev = torch.arange(Vd, dtype=torch.int32, device=DEV)
    h_g = to_dev_bf16(synth.gen_h(60, 1, H))
    h_e = to_dev_bf16(synth.gen_h(61, 1, H))
    alone = {}
    for name, h in (("g", h_g), ("e", h_e)):
        a, b = vt.vt_draft_head(h, W_dev, d2t_dev, k)
        torch.cuda.synchronize()
        alone[name] = (a.cpu().numpy(), b.cpu().numpy())
    need = vt.vt_draft_head_workspace_bytes(1, H, Vd, k)
    ws_g, ws_e = vt.new_workspace(need, DEV), vt.new_workspace(need, DEV)
    ids_g = torch.empty((1, k), dtype=torch.int32, device=DEV)
    lp_g = torch.empty((1, k), dtype=torch.float32, device=DEV)
    n_eager = 1100
    ids_e = torch.empty((n_eager, 1, k), dtype=torch.int32, device=DEV)
    lp_e = torch.empty((n_eager, 1, k), dtype=torch.float32, device=DEV)
    s_g, s_e = torch.cuda.Stream(), torch.cuda.Stream()  # default priority
    torch.cuda.synchronize()
    with torch.cuda.stream(s_g):
        vt.vt_draft_head(h_g, W_dev, d2t_dev, k, ids_g, lp_g, ws_g)  # warm: one-time kernel attributes
        s_g.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s_g):
            vt.vt_draft_head(h_g, W_dev, d2t_dev, k, ids_g, lp_g, ws_g)
    torch.cuda.synchronize()
    n_replay, bad = 60, 0
    for rep in range(n_replay):
        with torch.cuda.stream(s_g):
            ids_g.fill_(-7)
            g.replay()
        with torch.cuda.stream(s_e):
            lo, hi = rep * n_eager // n_replay, (rep + 1) * n_eager // n_replay
            for n in range(lo, hi):
                vt.vt_draft_head(h_e, W_dev, d2t_dev, k, ids_e[n], lp_e[n], ws_e)
        if rep % 10 == 9:
            s_g.synchronize()
            bad += int(not np.array_equal(ids_g.cpu().numpy(), alone["g"][0]))
            bad += int(not np.array_equal(lp_g.cpu().numpy().view(np.uint32), alone["g"][1].view(np.uint32)))
    torch.cuda.synchronize()
    assert bad == 0
    assert np.array_equal(ids_g.cpu().numpy(), alone["g"][0])
    e_ids, e_lp = ids_e.cpu().numpy(), lp_e.cpu().numpy()
    assert np.all(e_ids == alone["e"][0][None]) and np.all(e_lp.view(np.uint32) == alone["e"][1].view(np.uint32)[None])


# ------------------------------------------------------------------ full-size workloads
@pytest.fixture(scope="module")
def W2048():
    _say("generating W[128256,2048]")
    W = synth.gen_W(0, synth.FULL_VOCAB, 2048)
    return W, to_dev_bf16(W)


@pytest.fixture(scope="module")
def W4096():
    _say("generating W[128256,4096]")
    W = synth.gen_W(0, synth.FULL_VOCAB, 4096)
    return W, to_dev_bf16(W)


def _subset(W_pair, Vd):
    W, W_dev = W_pair
    ids = synth.zipf_subset(0, synth.FULL_VOCAB, Vd)
    ids_dev = torch.from_numpy(ids).to(DEV)
    Wsub_dev, d2t_dev = vt.vt_build_subset(W_dev, ids_dev)
    torch.cuda.synchronize()
    # gather parity at full size: d2t and every row of W_sub, bit for bit (in slabs, to bound host memory)
    assert np.array_equal(d2t_dev.cpu().numpy(), ids)
    Wsub_o, d2t_o = vo.build_subset(W, ids)
    assert np.array_equal(d2t_o, ids)
    slab = 16384
    for a in range(0, Vd, slab):
        assert np.array_equal(dev_bits(Wsub_dev[a:a + slab]), Wsub_o[a:a + slab]), "W_sub rows %d.." % a
    return ids, Wsub_dev, d2t_dev


def test_cfg0_trimmed_head_one_row(W2048):
    ids, Wsub_dev, d2t_dev = _subset(W2048, 4096)
    h = synth.gen_h(0, 1, 2048)
    g_ids, g_lp, g_z, g_lse = run_gpu(h, Wsub_dev, d2t_dev, 1)
    ora = vo.draft_head(h, W2048[0][ids], ids, 1)
    _say("cfg0 %s" % check_head(g_ids, g_lp, ora, ids, gpu_logits=g_z, gpu_lse=g_lse))


@pytest.mark.parametrize("B", [1, 4, 8])
def test_cfg1_untrimmed_baseline_head(W2048, B):
    ids, Wsub_dev, d2t_dev = _subset(W2048, synth.FULL_VOCAB)
    h = synth.gen_h(0, B, 2048)
    g_ids, g_lp, g_z, g_lse = run_gpu(h, Wsub_dev, d2t_dev, 10)
    ora = vo.draft_head(h, W2048[0], ids, 10)
    _say("cfg1 B=%d %s" % (B, check_head(g_ids, g_lp, ora, ids, gpu_logits=g_z, gpu_lse=g_lse)))


@pytest.mark.parametrize("Vd", [4096, 8192, 16384, 32768, 65536, 128256])
def test_cfg2_vocab_sweep(W4096, Vd):
    ids, Wsub_dev, d2t_dev = _subset(W4096, Vd)
    h = synth.gen_h(0, 1, 4096)
    g_ids, g_lp, g_z, g_lse = run_gpu(h, Wsub_dev, d2t_dev, 10)
    ora = vo.draft_head(h, W4096[0][ids], ids, 10)
    _say("cfg2 Vd=%d %s" % (Vd, check_head(g_ids, g_lp, ora, ids, gpu_logits=g_z, gpu_lse=g_lse)))


@pytest.mark.parametrize("rows,Vd,k", [(8, 13264, 8), (32, 13264, 8), (16, synth.FULL_VOCAB, 10), (32, synth.FULL_VOCAB, 10)])
def test_tree_step_of_a_few_rows_full_size(W4096, rows, Vd, k):
    """The tree-drafting steps bench.py times (8 and 32 nodes over the vocabulary Section 2.6 selects) and
    the kernel for a few rows over the whole vocabulary, one and two groups of rows: every logit, lse, id
    and log-probability against the oracle."""
    ids, Wsub_dev, d2t_dev = _subset(W4096, Vd)
    h = synth.gen_h(0, rows, 4096)
    assert vt.vt_draft_head_regime(rows, 4096, Vd, k) == 0
    g_ids, g_lp, g_z, g_lse = run_gpu(h, Wsub_dev, d2t_dev, k)
    ora = vo.draft_head(h, W4096[0] if Vd == synth.FULL_VOCAB else W4096[0][ids], ids, k)
    _say("tree step rows=%d Vd=%d %s" % (rows, Vd, check_head(g_ids, g_lp, ora, ids, gpu_logits=g_z, gpu_lse=g_lse)))
    n_ids, n_lp, _, _ = run_gpu(h, Wsub_dev, d2t_dev, k, debug=False)   # the timed entry point
    assert np.array_equal(n_ids, g_ids) and np.array_equal(n_lp, g_lp)


def _all_rows_check(name, W_pair, Vd, rows, k, peaked, chunk=64, logits_block=(0, 256)):
    """Every row of a tree-drafting-size batch against the oracle: ids (near-tie rule) and
    log-probs from the launch configuration that is timed (all rows in one call, no logits
    stored); plus, through the test hook, every logit and lse of one block of rows that spans a
    whole row tile of the matrix-core kernel, at full H and full V_draft."""
    ids, Wsub_dev, d2t_dev = _subset(W_pair, Vd)
    W_sub_host = W_pair[0] if Vd == synth.FULL_VOCAB else W_pair[0][ids]
    h = synth.gen_h(0, rows, 4096, peaked_frac=peaked)
    g_ids, g_lp, _, _ = run_gpu(h, Wsub_dev, d2t_dev, k, debug=False)
    worst = dict(max_dlogp=0.0, id_mismatch=0, id_mismatch_tight=0)
    for a in range(0, rows, chunk):   # the oracle in row chunks: bounds the host memory of its logits
        b = min(rows, a + chunk)
        ora = vo.draft_head(h[a:b], W_sub_host, ids, k)
        st = check_head(g_ids[a:b], g_lp[a:b], ora, ids)
        worst["max_dlogp"] = max(worst["max_dlogp"], st["max_dlogp"])
        worst["id_mismatch"] += st["id_mismatch"]
        worst["id_mismatch_tight"] += st["id_mismatch_tight"]
        _say("%s rows %d..%d ok" % (name, a, b - 1))
    _say("%s all %d rows: %s" % (name, rows, worst))
    assert worst["id_mismatch_tight"] == 0
    # the peaked rows are among them
    if peaked > 0:
        assert len(synth.peaked_rows(0, rows, peaked)) == int(peaked * rows)
    # logits and lse of a block of rows, at full size, through the test hook (same kernels)
    lo, hi = logits_block
    hb = h[lo:hi]
    b_ids, b_lp, b_z, b_lse = run_gpu(hb, Wsub_dev, d2t_dev, k, debug=True)
    for a in range(0, hi - lo, chunk):
        b = min(hi - lo, a + chunk)
        ora = vo.draft_head(hb[a:b], W_sub_host, ids, k)
        st = check_head(b_ids[a:b], b_lp[a:b], ora, ids, gpu_logits=b_z[a:b], gpu_lse=b_lse[a:b])
    _say("%s logits block rows %d..%d: %s" % (name, lo, hi - 1, st))
    # a block of rows on its own gives what the same rows give inside the full batch
    assert np.array_equal(b_ids, g_ids[lo:hi])
    assert np.max(np.abs(b_lp - g_lp[lo:hi])) <= 1e-5


def test_cfg3_tree_drafting_batch(W4096):
    _all_rows_check("cfg3", W4096, 32000, 1024, 8, 0.0)


def test_cfg4_large_batch_full_vocab(W4096):
    _all_rows_check("cfg4", W4096, synth.FULL_VOCAB, 512, 16, 0.05)
