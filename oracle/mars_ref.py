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
                      ("prob_ratio", "<f8"), ("gap", "<f8"),
                      ("id1", "<i4"), ("id2", "<i4"), ("relax_ok", "<i4"), ("relax_ok64", "<i4")],
                     align=True)
MARGIN_ROW_DTYPE = np.dtype([("z1", "<f8"), ("z2", "<f8"), ("ratio", "<f8"), ("prob_ratio", "<f8")])

# Indicators of a low margin (Sec. 3.3): logit ratio (Eq. 4), probability ratio, fixed logit margin.
IND_LOGIT_RATIO, IND_PROB_RATIO, IND_LOGIT_GAP = 0, 1, 2
DIAG_DTYPE = np.dtype([("bonus_prob", "<f8"), ("last_residual_norm", "<f8"),
                       ("min_accept_margin", "<f8"), ("min_cdf_margin", "<f8"), ("min_norm", "<f8"),
                       ("residual_passes", "<i4"), ("last_node", "<i4"),
                       ("small_norm_plen", "<i4"), ("small_norm_node", "<i4")], align=True)


def lib():
    global _LIB
    if _LIB is None:
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        L.mars_ref_row_stats.restype = ctypes.c_int
        L.mars_ref_verify.restype = ctypes.c_int
        L.mars_ref_row_stats_ex.restype = ctypes.c_int
        L.mars_ref_verify_ex.restype = ctypes.c_int
        L.mars_ref_commit.restype = ctypes.c_int
        L.mars_ref_margin_stats.restype = ctypes.c_int
        assert L.mars_ref_sizeof_row() == ROW_DTYPE.itemsize
        assert L.mars_ref_sizeof_diag() == DIAG_DTYPE.itemsize
        _LIB = L
    return _LIB


def set_norm_floor(z: float) -> None:
    """Residual normalisers below ``z`` are reported in diag's small_norm_plen / small_norm_node (no result changes)."""
    lib().mars_ref_set_norm_floor(ctypes.c_double(float(z)))


def get_norm_floor() -> float:
    L = lib()
    L.mars_ref_get_norm_floor.restype = ctypes.c_double
    return float(L.mars_ref_get_norm_floor())


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


def row_stats(logits, theta, temperature, indicator=IND_LOGIT_RATIO):
    """Per-row top-2, low-margin test and sum-exp.  Returns a structured array [B,N]."""
    logits = np.ascontiguousarray(logits)
    B, N, V = logits.shape
    th = _theta_array(theta, B)
    out = np.zeros((B, N), dtype=ROW_DTYPE)
    rc = lib().mars_ref_row_stats_ex(_ptr(logits), ctypes.c_int(_dtype_code(logits)), _ptr(th),
                                     ctypes.c_float(float(temperature)), ctypes.c_int(int(indicator)),
                                     ctypes.c_int(B), ctypes.c_int(N), ctypes.c_int(V), _ptr(out))
    if rc:
        raise ValueError(f"mars_ref_row_stats failed with {rc}")
    return out


def verify(logits, draft_tokens, tree_parent, theta, temperature, uniforms=None, draft_probs=None,
           indicator=IND_LOGIT_RATIO):
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
    rc = lib().mars_ref_verify_ex(
        _ptr(logits), ctypes.c_int(_dtype_code(logits)), _ptr(tok), _ptr(par),
        _ptr(dp), ctypes.c_int(dcode), _ptr(th), ctypes.c_float(float(temperature)), _ptr(u),
        ctypes.c_int(B), ctypes.c_int(N), ctypes.c_int(V), ctypes.c_int(int(indicator)),
        _ptr(out["accept_mask"]), _ptr(out["accept_len"]), _ptr(out["path_idx"]),
        _ptr(out["bonus_token"]), _ptr(out["decision"]), _ptr(out["request_status"]),
        _ptr(out["stats"]), _ptr(out["diag"]))
    if rc:
        raise ValueError(f"mars_ref_verify failed with {rc}")
    return out


def commit(draft_tokens, accept_len, path_idx, bonus_token):
    """Alg. 1's V_out per request (accepted draft tokens then the correction / bonus token, -1 padded)
    and the flat cache rows that stay (root and accepted nodes, request by request, path order)."""
    tok = np.ascontiguousarray(draft_tokens, dtype=np.int32)
    B, N = tok.shape
    ln = np.ascontiguousarray(accept_len, dtype=np.int32)
    path = np.ascontiguousarray(path_idx, dtype=np.int32)
    bonus = np.ascontiguousarray(bonus_token, dtype=np.int32)
    out = {"out_tokens": np.zeros((B, N), np.int32), "out_len": np.zeros((B,), np.int32),
           "keep_rows": np.zeros((B * N,), np.int32), "keep_offsets": np.zeros((B + 1,), np.int32)}
    rc = lib().mars_ref_commit(_ptr(tok), _ptr(ln), _ptr(path), _ptr(bonus), ctypes.c_int(B), ctypes.c_int(N),
                               _ptr(out["out_tokens"]), _ptr(out["out_len"]), _ptr(out["keep_rows"]),
                               _ptr(out["keep_offsets"]))
    if rc:
        raise ValueError(f"mars_ref_commit failed with {rc}")
    return out


def verify_sweep(logits, draft_tokens, tree_parent, thetas, temperature, uniforms=None, draft_probs=None,
                 indicator=IND_LOGIT_RATIO):
    """The pass repeated for each row of thresholds thetas[K,B] (the threshold ablation of Sec. 4):
    every output gains a leading axis of length K.  By definition K independent runs."""
    th = np.asarray(thetas, dtype=np.float32)
    assert th.ndim == 2
    runs = [verify(logits, draft_tokens, tree_parent, th[k], temperature, uniforms, draft_probs, indicator)
            for k in range(th.shape[0])]
    return {key: np.stack([r[key] for r in runs]) for key in runs[0]}


def margin_stats(logits, theta, temperature, ranges, bins):
    """Top-2 statistics per row and their histograms.  ranges = ((lo,hi) of z1, of z2/z1, of p2/p1),
    bins = three cell counts.  Histograms have bins+2 counters (below lo, the cells, at or above hi)."""
    logits = np.ascontiguousarray(logits)
    B, N, V = logits.shape
    th = _theta_array(theta, B)
    rg = np.ascontiguousarray(np.asarray(ranges, dtype=np.float32).reshape(6))
    bn = np.ascontiguousarray(np.asarray(bins, dtype=np.int32).reshape(3))
    out = {"rows": np.zeros((B, N), dtype=MARGIN_ROW_DTYPE),
           "hist_z1": np.zeros((int(bn[0]) + 2,), np.uint32),
           "hist_ratio": np.zeros((int(bn[1]) + 2,), np.uint32),
           "hist_prob": np.zeros((int(bn[2]) + 2,), np.uint32),
           "summary": np.zeros((4,), np.uint32),
           "edge_dist": np.zeros((B, N), np.float64)}
    rc = lib().mars_ref_margin_stats(_ptr(logits), ctypes.c_int(_dtype_code(logits)), _ptr(th),
                                     ctypes.c_float(float(temperature)), ctypes.c_int(B), ctypes.c_int(N),
                                     ctypes.c_int(V), _ptr(rg), _ptr(bn), _ptr(out["rows"]), _ptr(out["hist_z1"]),
                                     _ptr(out["hist_ratio"]), _ptr(out["hist_prob"]), _ptr(out["summary"]),
                                     _ptr(out["edge_dist"]))
    if rc:
        raise ValueError(f"mars_ref_margin_stats failed with {rc}")
    return out
