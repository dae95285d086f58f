"""The allocation-free entry point (device-resident scratch inside the library) against the
workspace entry point: same kernels, so ids and log-probs must be equal bit for bit; two calls in
a row per regime, the second with a smaller input (the scratch keeps the first call's partial
results), and sizes beyond the scratch capacity are refused."""
import numpy as np
import pytest
import torch

import paper_2603_05210_amd as vt
from paper_2603_05210_amd import synth
from tests.parity_util import to_dev_bf16

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _pair(seed, rows, H, Vd, k, W_dev):
    h = to_dev_bf16(synth.gen_h(seed, rows, H))
    d2t = (torch.arange(Vd, dtype=torch.int32, device=DEV) * 2 + 1).contiguous()
    W = W_dev[:Vd].contiguous()
    want_ids, want_lp = vt.vt_draft_head(h, W, d2t, k)
    torch.cuda.synchronize()
    ids = torch.full((rows, k), -9, dtype=torch.int32, device=DEV)
    lp = torch.full((rows, k), float("nan"), dtype=torch.float32, device=DEV)
    before = torch.cuda.memory_allocated()
    vt.vt_draft_head_static(h, W, d2t, k, ids, lp)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert np.array_equal(ids.cpu().numpy(), want_ids.cpu().numpy()), (rows, H, Vd, k)
    assert np.array_equal(lp.cpu().numpy().view(np.uint32), want_lp.cpu().numpy().view(np.uint32)), (rows, H, Vd, k)


@pytest.mark.parametrize("first,second", [
    ((1, 1024, 30011, 10), (1, 1024, 4099, 3)),      # single-launch merge: arrival counter reused
    ((2, 1024, 30011, 16), (1, 1024, 700, 1)),
    ((8, 1024, 30011, 10), (5, 1024, 9001, 4)),      # streaming + merge kernel
    ((300, 1024, 5000, 8), (40, 1024, 1300, 16)),    # matrix-core regime
])
def test_static_scratch_entry_matches_workspace_entry(first, second):
    print("no-alloc case", first, second, flush=True)
    W_dev = to_dev_bf16(synth.gen_W(91, 30011, 1024, std=0.05))
    for n, (rows, H, Vd, k) in enumerate((first, second, first)):
        _pair(100 + n, rows, H, Vd, k, W_dev)


def test_sizes_beyond_the_scratch_capacity_are_refused():
    rows, H, Vd, k = 2048, 64, 128256, 64
    assert vt.vt_draft_head_workspace_bytes(rows, H, Vd, k) > vt.VT_STATIC_SCRATCH_BYTES
    st = vt.lib().vt_draft_head_static(0x1000, rows, H, 0x1000, 0x1000, Vd, k, 0x1000, 0x1000, None)
    assert st == 6
    st = vt.lib().vt_draft_head_static(None, 1, 64, 0x1000, 0x1000, 100, 1, 0x1000, 0x1000, None)
    assert st == 1
