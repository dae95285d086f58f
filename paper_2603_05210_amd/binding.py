"""Thin Python binding of the C ABI in include/vt.h: argument marshalling only.

Tensors are torch tensors used purely as device memory (bf16 data may be torch.bfloat16 or a
16-bit integer view of the same bits); the current torch stream is passed as the HIP stream.
Every step of the head runs inside libvt.so.  There is no fallback: if the library is missing
or cannot be loaded, importing callers get an error.
"""
from __future__ import annotations

import ctypes
from pathlib import Path

import torch

_PKG = Path(__file__).resolve().parent
LIB_PATH = _PKG / "libvt.so"

VT_OK = 0
VT_MAX_K = 64
VT_WORKSPACE_HEADER_BYTES = 8192
STATUS_NAMES = {
    0: "VT_OK", 1: "VT_ERR_NULL", 2: "VT_ERR_SHAPE", 3: "VT_ERR_K", 4: "VT_ERR_ID_RANGE",
    5: "VT_ERR_ID_DUP", 6: "VT_ERR_WORKSPACE", 7: "VT_ERR_ALIGN", 8: "VT_ERR_DEVICE",
}

# every symbol include/vt.h declares
EXPORTS = (
    "vt_version", "vt_status_str", "vt_build_subset", "vt_check_token_ids_host",
    "vt_validate_build_subset_args", "vt_validate_draft_head_args", "vt_draft_head_workspace_bytes",
    "vt_draft_head_workspace_init", "vt_draft_head_regime", "vt_draft_head", "vt_draft_head_debug",
    "vt_draft_head_static", "vt_subset_q_code_bytes", "vt_subset_q_scale_bytes", "vt_build_subset_q",
    "vt_draft_head_q_workspace_bytes", "vt_draft_head_q", "vt_draft_head_q_debug", "vt_feature_fusion",
    "vt_draft_head_fused_workspace_bytes", "vt_draft_head_fused", "vt_draft_head_fused_debug",
    "vt_select_vocab_workspace_bytes", "vt_validate_select_vocab_args",
    "vt_select_vocab", "vt_build_t2d", "vt_coverage_workspace_bytes", "vt_coverage",
)


class VtError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s" % (where, status_str(status)))


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library.  Raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not LIB_PATH.exists():
            raise RuntimeError("%s is missing: build it with `python -m paper_2603_05210_amd.build` "
                               "(or __graft_entry__.build())" % LIB_PATH)
        L = ctypes.CDLL(str(LIB_PATH))
        p, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t
        L.vt_version.restype = i32
        L.vt_status_str.restype = ctypes.c_char_p
        L.vt_status_str.argtypes = [i32]
        L.vt_build_subset.restype = i32
        L.vt_build_subset.argtypes = [p, i64, i64, p, i64, p, p, p]
        L.vt_check_token_ids_host.restype = i32
        L.vt_check_token_ids_host.argtypes = [p, i64, i64]
        L.vt_validate_build_subset_args.restype = i32
        L.vt_validate_build_subset_args.argtypes = [p, i64, i64, p, i64, p, p]
        L.vt_validate_draft_head_args.restype = i32
        L.vt_validate_draft_head_args.argtypes = [p, i64, i64, p, p, i64, i32, p, p, p, sz]
        L.vt_draft_head_workspace_bytes.restype = sz
        L.vt_draft_head_workspace_bytes.argtypes = [i64, i64, i64, i32]
        L.vt_draft_head_regime.restype = i32
        L.vt_draft_head_regime.argtypes = [i64, i64, i64, i32]
        L.vt_draft_head.restype = i32
        L.vt_draft_head.argtypes = [p, i64, i64, p, p, i64, i32, p, p, p, sz, p]
        L.vt_draft_head_static.restype = i32
        L.vt_draft_head_static.argtypes = [p, i64, i64, p, p, i64, i32, p, p, p]
        L.vt_subset_q_code_bytes.restype = sz
        L.vt_subset_q_code_bytes.argtypes = [i32, i64, i64]
        L.vt_subset_q_scale_bytes.restype = sz
        L.vt_subset_q_scale_bytes.argtypes = [i32, i64, i64]
        L.vt_build_subset_q.restype = i32
        L.vt_build_subset_q.argtypes = [p, i64, i64, p, i64, i32, p, p, p, p]
        L.vt_draft_head_q_workspace_bytes.restype = sz
        L.vt_draft_head_q_workspace_bytes.argtypes = [i32, i64, i64, i64, i32]
        L.vt_draft_head_q.restype = i32
        L.vt_draft_head_q.argtypes = [p, i64, i64, p, p, i32, p, i64, i32, p, p, p, sz, p]
        L.vt_draft_head_q_debug.restype = i32
        L.vt_draft_head_q_debug.argtypes = [p, i64, i64, p, p, i32, p, i64, i32, p, p, p, sz, p, p, p]
        L.vt_feature_fusion.restype = i32
        L.vt_feature_fusion.argtypes = [p, i64, i64, p, i64, p, p]
        L.vt_draft_head_fused_workspace_bytes.restype = sz
        L.vt_draft_head_fused_workspace_bytes.argtypes = [i64, i64, i64, i32]
        L.vt_draft_head_fused.restype = i32
        L.vt_draft_head_fused.argtypes = [p, p, ctypes.c_float, p, i64, i64, p, p, i64, i32, p, p, p, sz, p]
        L.vt_draft_head_fused_debug.restype = i32
        L.vt_draft_head_fused_debug.argtypes = [p, p, ctypes.c_float, p, i64, i64, p, p, i64, i32, p, p, p, sz, p, p, p, p]
        L.vt_draft_head_debug.restype = i32
        L.vt_draft_head_debug.argtypes = [p, i64, i64, p, p, i64, i32, p, p, p, sz, p, p, p]
        L.vt_draft_head_workspace_init.restype = i32
        L.vt_draft_head_workspace_init.argtypes = [p, sz, p]
        f64 = ctypes.c_double
        L.vt_select_vocab_workspace_bytes.restype = sz
        L.vt_select_vocab_workspace_bytes.argtypes = [i64]
        L.vt_validate_select_vocab_args.restype = i32
        L.vt_validate_select_vocab_args.argtypes = [p, i64, i64, i64, f64, f64, f64, i64, i64, p, p, p, p, p, sz]
        L.vt_select_vocab.restype = i32
        L.vt_select_vocab.argtypes = [p, i64, i64, i64, f64, f64, f64, i64, i64, p, p, p, p, p, sz, p]
        L.vt_coverage_workspace_bytes.restype = sz
        L.vt_coverage_workspace_bytes.argtypes = [i64]
        L.vt_build_t2d.restype = i32
        L.vt_build_t2d.argtypes = [p, i64, i64, p, p, sz, p]
        L.vt_coverage.restype = i32
        L.vt_coverage.argtypes = [p, i64, p, i64, p, p, p, sz, p]
        _lib = L
    return _lib


def status_str(status: int) -> str:
    return lib().vt_status_str(int(status)).decode()


def _stream_ptr(t: torch.Tensor) -> int:
    return torch.cuda.current_stream(t.device).cuda_stream


def _dev16(t: torch.Tensor, name: str) -> torch.Tensor:
    if not t.is_cuda or not t.is_contiguous() or t.element_size() != 2:
        raise TypeError("%s must be a contiguous 16-bit device tensor (bf16 bits)" % name)
    return t


def _devi32(t: torch.Tensor, name: str) -> torch.Tensor:
    if not t.is_cuda or not t.is_contiguous() or t.dtype != torch.int32:
        raise TypeError("%s must be a contiguous int32 device tensor" % name)
    return t


def vt_version() -> int:
    return int(lib().vt_version())


def vt_draft_head_workspace_bytes(rows: int, H: int, V_draft: int, k: int) -> int:
    return int(lib().vt_draft_head_workspace_bytes(rows, H, V_draft, k))


def vt_draft_head_regime(rows: int, H: int, V_draft: int, k: int) -> int:
    return int(lib().vt_draft_head_regime(rows, H, V_draft, k))


def vt_check_token_ids_host(ids_host, V: int) -> int:
    """Status code for a host array of ids against vocabulary size V (touches no device)."""
    import numpy as np
    a = np.ascontiguousarray(ids_host, dtype=np.int32)
    return int(lib().vt_check_token_ids_host(a.ctypes.data_as(ctypes.c_void_p), a.shape[0], V))


def vt_build_subset(full_W: torch.Tensor, token_ids: torch.Tensor, W_sub_out: torch.Tensor | None = None,
                    d2t_out: torch.Tensor | None = None):
    """W_sub[V_draft,H], d2t[V_draft] for the draft vocabulary `token_ids` (device int32)."""
    _dev16(full_W, "full_W")
    _devi32(token_ids, "token_ids")
    V, H = full_W.shape
    Vd = token_ids.shape[0]
    if W_sub_out is None:
        W_sub_out = torch.empty((Vd, H), dtype=full_W.dtype, device=full_W.device)
    if d2t_out is None:
        d2t_out = torch.empty((Vd,), dtype=torch.int32, device=full_W.device)
    _dev16(W_sub_out, "W_sub_out")
    _devi32(d2t_out, "d2t_out")
    with torch.cuda.device(full_W.device):
        st = lib().vt_build_subset(full_W.data_ptr(), V, H, token_ids.data_ptr(), Vd, W_sub_out.data_ptr(),
                                   d2t_out.data_ptr(), _stream_ptr(full_W))
    if st != VT_OK:
        raise VtError(st, "vt_build_subset")
    return W_sub_out, d2t_out


def vt_draft_head_workspace_init(workspace: torch.Tensor) -> torch.Tensor:
    """Prepare a freshly allocated workspace buffer for vt_draft_head (zeroes its header)."""
    if not workspace.is_cuda or not workspace.is_contiguous():
        raise TypeError("workspace must be a contiguous device tensor")
    with torch.cuda.device(workspace.device):
        st = lib().vt_draft_head_workspace_init(workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                                _stream_ptr(workspace))
    if st != VT_OK:
        raise VtError(st, "vt_draft_head_workspace_init")
    return workspace


def new_workspace(nbytes: int, device) -> torch.Tensor:
    """A device buffer of at least `nbytes` bytes, initialised for vt_draft_head."""
    return vt_draft_head_workspace_init(torch.empty(max(int(nbytes), VT_WORKSPACE_HEADER_BYTES), dtype=torch.uint8, device=device))


class Workspace:
    """A reusable device buffer sized by vt_draft_head_workspace_bytes (initialised when it grows)."""

    def __init__(self, device):
        self.device = device
        self.buf = None

    def get(self, nbytes: int) -> torch.Tensor:
        if self.buf is None or self.buf.numel() < nbytes:
            self.buf = new_workspace(nbytes, self.device)
        return self.buf


def vt_draft_head(h: torch.Tensor, W_sub: torch.Tensor, d2t: torch.Tensor, k: int,
                  out_target_ids: torch.Tensor | None = None, out_logprobs: torch.Tensor | None = None,
                  workspace: torch.Tensor | None = None, logits_out: torch.Tensor | None = None,
                  lse_out: torch.Tensor | None = None):
    """One draft step: (target ids [rows,k] int32 best first, log-probs [rows,k] fp32).

    Passing logits_out / lse_out routes through vt_draft_head_debug (test hook).
    """
    _dev16(h, "h")
    _dev16(W_sub, "W_sub")
    _devi32(d2t, "d2t")
    rows, H = h.shape
    Vd, H2 = W_sub.shape
    if H2 != H or d2t.shape[0] != Vd:
        raise ValueError("shape mismatch between h, W_sub and d2t")
    dev = h.device
    if out_target_ids is None:
        out_target_ids = torch.empty((rows, k), dtype=torch.int32, device=dev)
    if out_logprobs is None:
        out_logprobs = torch.empty((rows, k), dtype=torch.float32, device=dev)
    need = vt_draft_head_workspace_bytes(rows, H, Vd, k)
    if workspace is None:
        workspace = new_workspace(need, dev)
    L = lib()
    with torch.cuda.device(dev):
        if logits_out is None and lse_out is None:
            st = L.vt_draft_head(h.data_ptr(), rows, H, W_sub.data_ptr(), d2t.data_ptr(), Vd, k,
                                 out_target_ids.data_ptr(), out_logprobs.data_ptr(), workspace.data_ptr(),
                                 workspace.numel(), _stream_ptr(h))
        else:
            st = L.vt_draft_head_debug(h.data_ptr(), rows, H, W_sub.data_ptr(), d2t.data_ptr(), Vd, k,
                                       out_target_ids.data_ptr(), out_logprobs.data_ptr(), workspace.data_ptr(),
                                       workspace.numel(), _stream_ptr(h),
                                       None if logits_out is None else logits_out.data_ptr(),
                                       None if lse_out is None else lse_out.data_ptr())
    if st != VT_OK:
        raise VtError(st, "vt_draft_head")
    return out_target_ids, out_logprobs


VT_STATIC_SCRATCH_BYTES = 40 << 20


def vt_draft_head_static(h: torch.Tensor, W_sub: torch.Tensor, d2t: torch.Tensor, k: int,
                         out_target_ids: torch.Tensor, out_logprobs: torch.Tensor):
    """vt_draft_head without a workspace argument and without any allocation: outputs must be
    passed in; partial results live in the library's device-resident scratch array."""
    _dev16(h, "h")
    _dev16(W_sub, "W_sub")
    _devi32(d2t, "d2t")
    _devi32(out_target_ids, "out_target_ids")
    rows, H = h.shape
    Vd, H2 = W_sub.shape
    if H2 != H or d2t.shape[0] != Vd:
        raise ValueError("shape mismatch between h, W_sub and d2t")
    if tuple(out_target_ids.shape) != (rows, k) or tuple(out_logprobs.shape) != (rows, k) or \
            out_logprobs.dtype != torch.float32 or not out_logprobs.is_contiguous():
        raise ValueError("outputs must be contiguous [rows,k] int32 / float32 device tensors")
    with torch.cuda.device(h.device):
        st = lib().vt_draft_head_static(h.data_ptr(), rows, H, W_sub.data_ptr(), d2t.data_ptr(), Vd, k,
                                        out_target_ids.data_ptr(), out_logprobs.data_ptr(), _stream_ptr(h))
    if st != VT_OK:
        raise VtError(st, "vt_draft_head_static")
    return out_target_ids, out_logprobs


def vt_feature_fusion(x: torch.Tensor, W_fc: torch.Tensor, g_out: torch.Tensor | None = None) -> torch.Tensor:
    """g[rows,d_out] = x[rows,d_in] . W_fc[d_out,d_in]^T (bf16 in and out, fp32 accumulation)."""
    _dev16(x, "x")
    _dev16(W_fc, "W_fc")
    rows, d_in = x.shape
    d_out, d_in2 = W_fc.shape
    if d_in2 != d_in:
        raise ValueError("shape mismatch between x and W_fc")
    if g_out is None:
        g_out = torch.empty((rows, d_out), dtype=x.dtype, device=x.device)
    with torch.cuda.device(x.device):
        st = lib().vt_feature_fusion(x.data_ptr(), rows, d_in, W_fc.data_ptr(), d_out, g_out.data_ptr(), _stream_ptr(x))
    if st != VT_OK:
        raise VtError(st, "vt_feature_fusion")
    return g_out


def vt_draft_head_fused_workspace_bytes(rows: int, H: int, V_draft: int, k: int) -> int:
    return int(lib().vt_draft_head_fused_workspace_bytes(rows, H, V_draft, k))


def vt_draft_head_fused(g: torch.Tensor, gamma: torch.Tensor, eps: float, W_sub: torch.Tensor, d2t: torch.Tensor, k: int,
                        parent_scores: torch.Tensor | None = None, out_target_ids: torch.Tensor | None = None,
                        out_scores: torch.Tensor | None = None, workspace: torch.Tensor | None = None,
                        logits_out: torch.Tensor | None = None, lse_out: torch.Tensor | None = None,
                        h_out: torch.Tensor | None = None):
    """RMSNorm -> draft head -> path scores in one call: (target ids [rows,k], scores [rows,k])."""
    _dev16(g, "g")
    _dev16(gamma, "gamma")
    _dev16(W_sub, "W_sub")
    _devi32(d2t, "d2t")
    rows, H = g.shape
    Vd = W_sub.shape[0]
    dev = g.device
    if out_target_ids is None:
        out_target_ids = torch.empty((rows, k), dtype=torch.int32, device=dev)
    if out_scores is None:
        out_scores = torch.empty((rows, k), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = new_workspace(vt_draft_head_fused_workspace_bytes(rows, H, Vd, k), dev)
    opt = lambda t: None if t is None else t.data_ptr()
    with torch.cuda.device(dev):
        st = lib().vt_draft_head_fused_debug(g.data_ptr(), gamma.data_ptr(), float(eps), opt(parent_scores), rows, H,
                                             W_sub.data_ptr(), d2t.data_ptr(), Vd, k, out_target_ids.data_ptr(),
                                             out_scores.data_ptr(), workspace.data_ptr(), workspace.numel(),
                                             _stream_ptr(g), opt(logits_out), opt(lse_out), opt(h_out))
    if st != VT_OK:
        raise VtError(st, "vt_draft_head_fused")
    return out_target_ids, out_scores


VT_Q_FP8_E4M3 = 1
VT_Q_MXFP4 = 2


def vt_build_subset_q(full_W: torch.Tensor, token_ids: torch.Tensor, fmt: int):
    """Compressed W_sub for the draft vocabulary `token_ids`: (codes uint8, scales, d2t) device tensors.
    FP8: codes [V_draft,H], scales float32 [V_draft]; MXFP4: codes [V_draft,H/2], scales uint8 [V_draft,H/32]."""
    _dev16(full_W, "full_W")
    _devi32(token_ids, "token_ids")
    V, H = full_W.shape
    Vd = token_ids.shape[0]
    L = lib()
    nc, ns = int(L.vt_subset_q_code_bytes(fmt, Vd, H)), int(L.vt_subset_q_scale_bytes(fmt, Vd, H))
    if nc == 0:
        raise VtError(2, "vt_build_subset_q")
    dev = full_W.device
    codes = torch.empty((Vd, nc // Vd), dtype=torch.uint8, device=dev)
    scales = (torch.empty((Vd,), dtype=torch.float32, device=dev) if fmt == VT_Q_FP8_E4M3
              else torch.empty((Vd, ns // Vd), dtype=torch.uint8, device=dev))
    d2t = torch.empty((Vd,), dtype=torch.int32, device=dev)
    with torch.cuda.device(dev):
        st = L.vt_build_subset_q(full_W.data_ptr(), V, H, token_ids.data_ptr(), Vd, fmt, codes.data_ptr(),
                                 scales.data_ptr(), d2t.data_ptr(), _stream_ptr(full_W))
    if st != VT_OK:
        raise VtError(st, "vt_build_subset_q")
    return codes, scales, d2t


def vt_draft_head_q_workspace_bytes(fmt: int, rows: int, H: int, V_draft: int, k: int) -> int:
    return int(lib().vt_draft_head_q_workspace_bytes(fmt, rows, H, V_draft, k))


def vt_draft_head_q(h: torch.Tensor, codes: torch.Tensor, scales: torch.Tensor, fmt: int, d2t: torch.Tensor, k: int,
                    out_target_ids: torch.Tensor | None = None, out_logprobs: torch.Tensor | None = None,
                    workspace: torch.Tensor | None = None, logits_out: torch.Tensor | None = None,
                    lse_out: torch.Tensor | None = None):
    """One draft step over a compressed W_sub (one row): (target ids [1,k], log-probs [1,k])."""
    _dev16(h, "h")
    _devi32(d2t, "d2t")
    if not (codes.is_cuda and codes.is_contiguous() and codes.dtype == torch.uint8 and scales.is_cuda
            and scales.is_contiguous()):
        raise TypeError("codes / scales must be contiguous device tensors")
    rows, H = h.shape
    Vd = codes.shape[0]
    dev = h.device
    if out_target_ids is None:
        out_target_ids = torch.empty((rows, k), dtype=torch.int32, device=dev)
    if out_logprobs is None:
        out_logprobs = torch.empty((rows, k), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = new_workspace(vt_draft_head_q_workspace_bytes(fmt, rows, H, Vd, k), dev)
    with torch.cuda.device(dev):
        st = lib().vt_draft_head_q_debug(h.data_ptr(), rows, H, codes.data_ptr(), scales.data_ptr(), fmt, d2t.data_ptr(),
                                         Vd, k, out_target_ids.data_ptr(), out_logprobs.data_ptr(),
                                         workspace.data_ptr(), workspace.numel(), _stream_ptr(h),
                                         None if logits_out is None else logits_out.data_ptr(),
                                         None if lse_out is None else lse_out.data_ptr())
    if st != VT_OK:
        raise VtError(st, "vt_draft_head_q")
    return out_target_ids, out_logprobs


class VtSelection(ctypes.Structure):
    """Mirror of vt_selection in include/vt.h."""
    _fields_ = [("k_star", ctypes.c_int64), ("feasible", ctypes.c_int32), ("C", ctypes.c_double),
                ("R", ctypes.c_double), ("U", ctypes.c_double), ("n_tokens", ctypes.c_uint64)]


def vt_select_vocab_workspace_bytes(V: int) -> int:
    return int(lib().vt_select_vocab_workspace_bytes(V))


def vt_select_vocab(tokens: torch.Tensor, V: int, d: int, F_fixed: float, alpha: float, c_min: float,
                    k_min: int, k_max: int, workspace: torch.Tensor | None = None):
    """Vocabulary-size selection over a device stream of token ids.  Returns (selection, freq[V]
    as int32 bit patterns of the uint32 counts, rank_ids[V], token_ids[k*]) -- device tensors."""
    _devi32(tokens, "tokens")
    dev = tokens.device
    freq = torch.empty(V, dtype=torch.int32, device=dev)
    rank_ids = torch.empty(V, dtype=torch.int32, device=dev)
    token_ids = torch.empty(V, dtype=torch.int32, device=dev)
    if workspace is None:
        workspace = torch.empty(max(16, vt_select_vocab_workspace_bytes(V)), dtype=torch.uint8, device=dev)
    res = VtSelection()
    st = lib().vt_select_vocab(tokens.data_ptr(), tokens.numel(), V, d, float(F_fixed), float(alpha), float(c_min),
                               k_min, k_max, freq.data_ptr(), rank_ids.data_ptr(), token_ids.data_ptr(),
                               ctypes.addressof(res), workspace.data_ptr(), workspace.numel(), _stream_ptr(tokens))
    if st != VT_OK:
        raise VtError(st, "vt_select_vocab")
    return res, freq, rank_ids, token_ids[: int(res.k_star)]


class VtCoverage(ctypes.Structure):
    """Mirror of vt_coverage_result in include/vt.h."""
    _fields_ = [("n_tokens", ctypes.c_uint64), ("n_covered", ctypes.c_uint64), ("n_unique", ctypes.c_uint64),
                ("n_unique_covered", ctypes.c_uint64), ("freq_coverage", ctypes.c_double),
                ("unique_coverage", ctypes.c_double)]


def vt_coverage_workspace_bytes(V: int) -> int:
    return int(lib().vt_coverage_workspace_bytes(V))


def vt_build_t2d(d2t: torch.Tensor, V: int, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """t2d[V] (device int32) from the draft-to-target buffer d2t[V_draft]."""
    _devi32(d2t, "d2t")
    t2d = torch.empty(V, dtype=torch.int32, device=d2t.device)
    if workspace is None:
        workspace = torch.empty(max(16, vt_coverage_workspace_bytes(V)), dtype=torch.uint8, device=d2t.device)
    st = lib().vt_build_t2d(d2t.data_ptr(), d2t.numel(), V, t2d.data_ptr(), workspace.data_ptr(), workspace.numel(),
                            _stream_ptr(d2t))
    if st != VT_OK:
        raise VtError(st, "vt_build_t2d")
    return t2d


def vt_coverage(tokens: torch.Tensor, t2d: torch.Tensor, want_draft_ids: bool = False,
                workspace: torch.Tensor | None = None):
    """Coverage counts and ratios of the vocabulary behind t2d on a device token stream; with
    want_draft_ids also the stream mapped through t2d.  Returns (VtCoverage, draft_ids or None)."""
    _devi32(tokens, "tokens")
    _devi32(t2d, "t2d")
    V = t2d.numel()
    if workspace is None:
        workspace = torch.empty(max(16, vt_coverage_workspace_bytes(V)), dtype=torch.uint8, device=tokens.device)
    out = torch.empty(tokens.numel(), dtype=torch.int32, device=tokens.device) if want_draft_ids else None
    res = VtCoverage()
    st = lib().vt_coverage(tokens.data_ptr(), tokens.numel(), t2d.data_ptr(), V,
                           out.data_ptr() if out is not None else None, ctypes.addressof(res),
                           workspace.data_ptr(), workspace.numel(), _stream_ptr(tokens))
    if st != VT_OK:
        raise VtError(st, "vt_coverage")
    return res, out
