"""TEST INFRASTRUCTURE -- ctypes access to the CPU oracle in vt_oracle.c.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this module; the
product package never does, and this module imports nothing from the product.  Arrays are
numpy: bf16 is carried as uint16 bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "vt_oracle.c"
_LIB = _HERE / "libvt_oracle.so"
_lib = None


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc (no fused multiply-add contraction, OpenMP over outputs)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(".so.tmp%d" % os.getpid())
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared", "-fPIC",
               "-std=c11", "-Wall", "-Wextra", str(_SRC), "-o", str(tmp), "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(str(_LIB))
        p = ctypes.c_void_p
        i64 = ctypes.c_int64
        lib.vto_num_threads.restype = ctypes.c_int
        lib.vto_build_subset.restype = ctypes.c_int
        lib.vto_build_subset.argtypes = [p, i64, i64, p, i64, p, p]
        lib.vto_logits.restype = None
        lib.vto_logits.argtypes = [p, i64, i64, p, i64, p, p]
        lib.vto_logits_f64.restype = None
        lib.vto_logits_f64.argtypes = [p, i64, i64, p, i64, p]
        lib.vto_lse_row.restype = ctypes.c_float
        lib.vto_lse_row.argtypes = [p, i64]
        lib.vto_topk_row.restype = None
        lib.vto_topk_row.argtypes = [p, i64, ctypes.c_int, p]
        lib.vto_draft_head.restype = ctypes.c_int
        lib.vto_draft_head.argtypes = [p, i64, i64, p, p, i64, ctypes.c_int, p, p, p, p, p, p]
        lib.vto_logits_w32.restype = None
        lib.vto_logits_w32.argtypes = [p, i64, i64, p, i64, p]
        lib.vto_draft_head_w32.restype = ctypes.c_int
        lib.vto_draft_head_w32.argtypes = [p, i64, i64, p, p, i64, ctypes.c_int, p, p, p, p, p]
        _lib = lib
    return _lib


def _ptr(a: np.ndarray | None):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, "bf16 is passed as uint16 bit patterns"
    return a


def num_threads() -> int:
    return int(_load().vto_num_threads())


def build_subset(W: np.ndarray, ids: np.ndarray):
    """(W_sub[Vd,H] uint16, d2t[Vd] int32) for the draft vocabulary `ids` (Section 2.1)."""
    W = _u16(W)
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    V, H = W.shape
    Vd = ids.shape[0]
    W_sub = np.empty((Vd, H), dtype=np.uint16)
    d2t = np.empty(Vd, dtype=np.int32)
    rc = _load().vto_build_subset(_ptr(W), V, H, _ptr(ids), Vd, _ptr(W_sub), _ptr(d2t))
    if rc == -1:
        raise ValueError("token id outside [0,V)")
    if rc == -2:
        raise ValueError("duplicate token id")
    if rc != 0:
        raise RuntimeError("oracle build_subset failed: %d" % rc)
    return W_sub, d2t


def logits(h: np.ndarray, W_sub: np.ndarray, return_flops: bool = False):
    """z[R,Vd] fp32 (Section 2.3 projection, sequential fp32 accumulation)."""
    h = _u16(h)
    W_sub = _u16(W_sub)
    R, H = h.shape
    Vd, H2 = W_sub.shape
    assert H == H2
    z = np.empty((R, Vd), dtype=np.float32)
    flops = ctypes.c_int64(0)
    _load().vto_logits(_ptr(h), R, H, _ptr(W_sub), Vd, _ptr(z), ctypes.byref(flops))
    return (z, int(flops.value)) if return_flops else z


def logits_f64(h: np.ndarray, W_sub: np.ndarray) -> np.ndarray:
    h = _u16(h)
    W_sub = _u16(W_sub)
    R, H = h.shape
    Vd = W_sub.shape[0]
    z = np.empty((R, Vd), dtype=np.float64)
    _load().vto_logits_f64(_ptr(h), R, H, _ptr(W_sub), Vd, _ptr(z))
    return z


def lse_row(z_row: np.ndarray) -> float:
    z_row = np.ascontiguousarray(z_row, dtype=np.float32)
    return float(_load().vto_lse_row(_ptr(z_row), z_row.shape[0]))


def topk_row(z_row: np.ndarray, k: int) -> np.ndarray:
    z_row = np.ascontiguousarray(z_row, dtype=np.float32)
    out = np.empty(k, dtype=np.int32)
    _load().vto_topk_row(_ptr(z_row), z_row.shape[0], k, _ptr(out))
    return out


class HeadResult:
    __slots__ = ("ids", "logp", "draft_idx", "z", "lse", "flops")


def draft_head(h: np.ndarray, W_sub: np.ndarray, d2t: np.ndarray, k: int, want_logits: bool = True) -> HeadResult:
    """The per-step head: target-vocabulary ids [R,k] best first and their log-probs over V_d."""
    h = _u16(h)
    W_sub = _u16(W_sub)
    d2t = np.ascontiguousarray(d2t, dtype=np.int32)
    R, H = h.shape
    Vd = W_sub.shape[0]
    assert W_sub.shape[1] == H and d2t.shape[0] == Vd
    res = HeadResult()
    res.ids = np.empty((R, k), dtype=np.int32)
    res.logp = np.empty((R, k), dtype=np.float32)
    res.draft_idx = np.empty((R, k), dtype=np.int32)
    res.z = np.empty((R, Vd), dtype=np.float32) if want_logits else None
    res.lse = np.empty(R, dtype=np.float32)
    flops = ctypes.c_int64(0)
    rc = _load().vto_draft_head(_ptr(h), R, H, _ptr(W_sub), _ptr(d2t), Vd, int(k), _ptr(res.ids),
                                _ptr(res.logp), _ptr(res.draft_idx), _ptr(res.z), _ptr(res.lse),
                                ctypes.byref(flops))
    if rc != 0:
        raise ValueError("k must be in [1, V_draft]")
    res.flops = int(flops.value)
    return res


def logits_w32(h: np.ndarray, W32: np.ndarray) -> np.ndarray:
    """z[R,Vd] fp32 for bf16 hidden states and fp32 weights (sequential fp32 accumulation)."""
    h = _u16(h)
    W32 = np.ascontiguousarray(W32, dtype=np.float32)
    R, H = h.shape
    Vd, H2 = W32.shape
    assert H == H2
    z = np.empty((R, Vd), dtype=np.float32)
    _load().vto_logits_w32(_ptr(h), R, H, _ptr(W32), Vd, _ptr(z))
    return z


def draft_head_w32(h: np.ndarray, W32: np.ndarray, d2t: np.ndarray, k: int, want_logits: bool = True) -> HeadResult:
    """The per-step head over fp32 weights (a dequantised compressed W_sub)."""
    h = _u16(h)
    W32 = np.ascontiguousarray(W32, dtype=np.float32)
    d2t = np.ascontiguousarray(d2t, dtype=np.int32)
    R, H = h.shape
    Vd = W32.shape[0]
    assert W32.shape[1] == H and d2t.shape[0] == Vd
    res = HeadResult()
    res.ids = np.empty((R, k), dtype=np.int32)
    res.logp = np.empty((R, k), dtype=np.float32)
    res.draft_idx = np.empty((R, k), dtype=np.int32)
    res.z = np.empty((R, Vd), dtype=np.float32) if want_logits else None
    res.lse = np.empty(R, dtype=np.float32)
    rc = _load().vto_draft_head_w32(_ptr(h), R, H, _ptr(W32), _ptr(d2t), Vd, int(k), _ptr(res.ids),
                                    _ptr(res.logp), _ptr(res.draft_idx), _ptr(res.z), _ptr(res.lse))
    if rc != 0:
        raise ValueError("k must be in [1, V_draft]")
    res.flops = 2 * R * H * Vd
    return res
