"""Host-only checks of the C-ABI library: it loads without a GPU, exports every symbol that
include/vt.h declares, and its argument validation returns the documented codes.  No kernel
is launched here."""
import ctypes
import re
from pathlib import Path

import numpy as np
import pytest

import paper_2603_05210_amd as vt

ROOT = Path(__file__).resolve().parent.parent
HEADER = (ROOT / "include" / "vt.h").read_text()


def _declared_functions():
    body = re.sub(r"/\*.*?\*/", "", HEADER, flags=re.S)
    names = re.findall(r"\b(vt_[a-z0-9_]+)\s*\(", body)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    L = vt.lib()
    declared = _declared_functions()
    assert len(declared) >= 10
    for name in declared:
        assert hasattr(L, name), name
    assert sorted(vt.EXPORTS) == declared


def test_version_and_status_strings():
    assert vt.vt_version() >= 100
    seen = set()
    for code in range(9):
        s = vt.status_str(code)
        assert s and s not in seen
        seen.add(s)
    assert vt.status_str(0) == "VT_OK"


FAKE = 0x1000  # a non-NULL, 16-byte aligned address; validation never dereferences it


def _validate_head(h=FAKE, rows=1, H=2048, W=FAKE, d2t=FAKE, Vd=4096, k=1, ids=FAKE, lp=FAKE, ws=FAKE, wsb=None):
    if wsb is None:
        wsb = max(vt.vt_draft_head_workspace_bytes(rows, H, Vd, k), 1)
    return vt.lib().vt_validate_draft_head_args(h, rows, H, W, d2t, Vd, k, ids, lp, ws, wsb)


def test_draft_head_argument_validation():
    assert _validate_head() == 0
    assert _validate_head(h=None) == 1
    assert _validate_head(W=None) == 1
    assert _validate_head(d2t=None) == 1
    assert _validate_head(ids=None) == 1
    assert _validate_head(lp=None) == 1
    assert _validate_head(rows=0) == 2
    assert _validate_head(H=2052) == 2
    assert _validate_head(H=0) == 2
    assert _validate_head(Vd=0) == 2
    assert _validate_head(k=0) == 3
    assert _validate_head(k=65) == 3
    assert _validate_head(Vd=8, k=9) == 3
    assert _validate_head(h=FAKE + 8) == 7
    assert _validate_head(W=FAKE + 2) == 7
    assert _validate_head(ws=None) == 6
    assert _validate_head(wsb=16) == 6
    assert _validate_head(ws=FAKE + 4) == 7


def test_build_subset_argument_validation():
    f = vt.lib().vt_validate_build_subset_args
    assert f(FAKE, 128256, 4096, FAKE, 32000, FAKE, FAKE) == 0
    assert f(None, 128256, 4096, FAKE, 32000, FAKE, FAKE) == 1
    assert f(FAKE, 128256, 4096, FAKE, 32000, FAKE, None) == 1
    assert f(FAKE, 100, 4096, FAKE, 101, FAKE, FAKE) == 2
    assert f(FAKE, 100, 4100, FAKE, 10, FAKE, FAKE) == 2
    assert f(FAKE, 0, 4096, FAKE, 0, FAKE, FAKE) == 2
    assert f(FAKE + 8, 100, 4096, FAKE, 10, FAKE, FAKE) == 7


def test_host_token_id_check():
    V = 1000
    assert vt.vt_check_token_ids_host(np.array([5, 1, 999], dtype=np.int32), V) == 0
    assert vt.vt_check_token_ids_host(np.array([5, 1000], dtype=np.int32), V) == 4
    assert vt.vt_check_token_ids_host(np.array([-1, 3], dtype=np.int32), V) == 4
    assert vt.vt_check_token_ids_host(np.array([7, 3, 7], dtype=np.int32), V) == 5
    assert vt.vt_check_token_ids_host(np.arange(V, dtype=np.int32), V) == 0
    assert vt.vt_check_token_ids_host(np.arange(V + 1, dtype=np.int32) % V, V) == 2


@pytest.mark.parametrize("rows,H,Vd,k,regime", [
    (1, 2048, 4096, 1, 0), (8, 2048, 128256, 10, 0), (16, 4096, 32000, 8, 0),
    (17, 4096, 32000, 8, 0), (32, 2048, 128256, 16, 0), (48, 4096, 13264, 10, 0), (48, 4096, 32000, 8, 1),
    (17, 4096, 32000, 17, 1), (17, 1024, 32000, 8, 1), (65, 4096, 4096, 8, 1),
    (1024, 4096, 32000, 8, 1), (512, 4096, 128256, 16, 1),
])
def test_regime_and_workspace_query(rows, H, Vd, k, regime):
    assert vt.vt_draft_head_regime(rows, H, Vd, k) == regime
    need = vt.vt_draft_head_workspace_bytes(rows, H, Vd, k)
    assert need > 0 and need % 256 == 0
    # the workspace holds partial results only: far below the fp32 logits it replaces for big shapes
    if rows * Vd > 1 << 22:
        assert need < 4 * rows * Vd
    assert vt.vt_draft_head_workspace_bytes(rows, H, Vd, 0) == 0
    assert vt.vt_draft_head_regime(rows, H + 1, Vd, k) == -1


def test_workspace_init_argument_validation():
    f = vt.lib().vt_draft_head_workspace_init
    assert f(None, 4096, None) == 1
    assert f(FAKE, 8191, None) == 6
    assert f(FAKE + 4, 1 << 20, None) == 7
    # every workspace size includes the header the call initialises
    assert vt.vt_draft_head_workspace_bytes(1, 64, 8, 1) >= 8192 + 256


def test_select_vocab_argument_validation():
    f = vt.lib().vt_validate_select_vocab_args
    V = 128256
    wsb = vt.vt_select_vocab_workspace_bytes(V)
    assert wsb >= (1 << 17) * 8 + V * 4
    assert vt.vt_select_vocab_workspace_bytes(0) == 0

    def call(tokens=FAKE, n=1000, V=V, d=4096, F=5.872e8, alpha=0.5, c_min=0.9, k_min=1024, k_max=V,
             freq=FAKE, rank=FAKE, ids=FAKE, res=FAKE, ws=FAKE, wsb=wsb):
        return f(tokens, n, V, d, F, alpha, c_min, k_min, k_max, freq, rank, ids, res, ws, wsb)

    assert call() == 0
    assert call(tokens=None) == 1 and call(res=None) == 1 and call(ids=None) == 1
    assert call(n=0) == 2 and call(n=1 << 32) == 2 and call(d=0) == 2
    assert call(alpha=1.5) == 2 and call(alpha=float("nan")) == 2 and call(c_min=-0.1) == 2 and call(F=-1.0) == 2
    assert call(k_min=0) == 3 and call(k_min=2000, k_max=1999) == 3 and call(k_max=V + 1) == 3
    assert call(ws=None) == 6 and call(wsb=wsb - 1) == 6
    assert call(tokens=FAKE + 4) == 7 and call(freq=FAKE + 2) == 7


def test_coverage_argument_validation():
    L = vt.lib()
    V = 128256
    wsb = vt.vt_coverage_workspace_bytes(V)
    assert wsb >= (V + 31) // 32 * 4 and vt.vt_coverage_workspace_bytes(0) == 0
    # host-side checks come first and never touch the pointers
    assert L.vt_build_t2d(None, 10, V, FAKE, FAKE, wsb, None) == 1
    assert L.vt_build_t2d(FAKE, 0, V, FAKE, FAKE, wsb, None) == 2
    assert L.vt_build_t2d(FAKE, V + 1, V, FAKE, FAKE, wsb, None) == 2
    assert L.vt_build_t2d(FAKE, 10, V, FAKE, None, 0, None) == 6
    assert L.vt_build_t2d(FAKE + 2, 10, V, FAKE, FAKE, wsb, None) == 7
    assert L.vt_coverage(None, 10, FAKE, V, None, FAKE, FAKE, wsb, None) == 1
    assert L.vt_coverage(FAKE, 10, FAKE, V, None, None, FAKE, wsb, None) == 1
    assert L.vt_coverage(FAKE, 0, FAKE, V, None, FAKE, FAKE, wsb, None) == 2
    assert L.vt_coverage(FAKE, 10, FAKE, V, None, FAKE, FAKE, wsb - 1, None) == 6
    assert L.vt_coverage(FAKE, 10, FAKE, V, FAKE + 1, FAKE, FAKE, wsb, None) == 7
