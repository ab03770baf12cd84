"""ctypes wrapper of the C oracle (oracle/mars_ref.c) -- test infrastructure only.

Arrays are numpy, on the host.  bf16 tensors are passed as ``uint16`` arrays holding
the bf16 bit patterns; fp32 tensors as ``float32``.  Nothing here touches the GPU
or the HIP library.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None

ROW_DTYPE = np.dtype([("z1", "<f8"), ("z2", "<f8"), ("ratio", "<f8"), ("sum_exp", "<f8"),
                      ("id1", "<i4"), ("id2", "<i4"), ("relax_ok", "<i4"), ("relax_ok64", "<i4")],
                     align=True)
DIAG_DTYPE = np.dtype([("bonus_prob", "<f8"), ("last_residual_norm", "<f8"),
                       ("min_accept_margin", "<f8"), ("min_cdf_margin", "<f8"), ("min_norm", "<f8"),
                       ("residual_passes", "<i4"), ("last_node", "<i4")], align=True)


def lib():
    global _LIB
    if _LIB is None:
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        L.mars_ref_row_stats.restype = ctypes.c_int
        L.mars_ref_verify.restype = ctypes.c_int
        assert L.mars_ref_sizeof_row() == ROW_DTYPE.itemsize
        assert L.mars_ref_sizeof_diag() == DIAG_DTYPE.itemsize
        _LIB = L
    return _LIB


def set_threads(n: int) -> None:
    lib().mars_ref_set_threads(ctypes.c_int(int(n)))


def get_threads() -> int:
    return int(lib().mars_ref_get_threads())


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return 0
    if a.dtype == np.uint16:
        return 1
    raise TypeError(f"logits/draft_probs must be float32 or uint16 (bf16 bits), got {a.dtype}")


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _theta_array(theta, B):
    t = np.asarray(theta, dtype=np.float32)
    if t.ndim == 0:
        t = np.full((B,), t, dtype=np.float32)
    assert t.shape == (B,)
    return np.ascontiguousarray(t)


def row_stats(logits, theta, temperature):
    """Per-row top-2, ratio test and sum-exp.  Returns a structured array [B,N]."""
    logits = np.ascontiguousarray(logits)
    B, N, V = logits.shape
    th = _theta_array(theta, B)
    out = np.zeros((B, N), dtype=ROW_DTYPE)
    rc = lib().mars_ref_row_stats(_ptr(logits), ctypes.c_int(_dtype_code(logits)), _ptr(th),
                                  ctypes.c_float(float(temperature)), ctypes.c_int(B),
                                  ctypes.c_int(N), ctypes.c_int(V), _ptr(out))
    if rc:
        raise ValueError(f"mars_ref_row_stats failed with {rc}")
    return out


def verify(logits, draft_tokens, tree_parent, theta, temperature, uniforms=None, draft_probs=None):
    """The whole verification pass on the CPU.  Returns a dict of numpy arrays."""
    logits = np.ascontiguousarray(logits)
    B, N, V = logits.shape
    tok = np.ascontiguousarray(draft_tokens, dtype=np.int32)
    par = np.ascontiguousarray(tree_parent, dtype=np.int32)
    assert tok.shape == (B, N) and par.shape == (B, N)
    th = _theta_array(theta, B)
    u = None
    if uniforms is not None:
        u = np.ascontiguousarray(uniforms, dtype=np.float32)
        assert u.shape == (B, N + 1)
    dp, dcode = None, 0
    if draft_probs is not None:
        dp = np.ascontiguousarray(draft_probs)
        assert dp.shape == (B, N, V)
        dcode = _dtype_code(dp)
    out = {
        "accept_mask": np.zeros((B, N), np.uint8),
        "accept_len": np.zeros((B,), np.int32),
        "path_idx": np.zeros((B, N), np.int32),
        "bonus_token": np.zeros((B,), np.int32),
        "decision": np.zeros((B, N), np.uint8),
        "request_status": np.zeros((B,), np.int32),
        "stats": np.zeros((B, N), dtype=ROW_DTYPE),
        "diag": np.zeros((B,), dtype=DIAG_DTYPE),
    }
    rc = lib().mars_ref_verify(
        _ptr(logits), ctypes.c_int(_dtype_code(logits)), _ptr(tok), _ptr(par),
        _ptr(dp), ctypes.c_int(dcode), _ptr(th), ctypes.c_float(float(temperature)), _ptr(u),
        ctypes.c_int(B), ctypes.c_int(N), ctypes.c_int(V),
        _ptr(out["accept_mask"]), _ptr(out["accept_len"]), _ptr(out["path_idx"]),
        _ptr(out["bonus_token"]), _ptr(out["decision"]), _ptr(out["request_status"]),
        _ptr(out["stats"]), _ptr(out["diag"]))
    if rc:
        raise ValueError(f"mars_ref_verify failed with {rc}")
    return out
