"""ctypes binding of libmars.so -- argument marshalling only.

The functions mirror include/mars.h name for name.  Tensors are torch CUDA tensors
(ROCm); bf16 logits may be given as ``torch.bfloat16`` or as ``torch.uint16``/``int16``
bit patterns.  Every call enqueues on the current torch stream and returns without
synchronising.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmars.so")

MARS_F32, MARS_BF16 = 0, 1
MARS_OK = 0
MARS_MAX_NODES = 1024
MARS_MAX_THETAS = 64
MARS_IND_LOGIT_RATIO, MARS_IND_PROB_RATIO, MARS_IND_LOGIT_GAP = 0, 1, 2
MARS_STAGE_ROWS, MARS_STAGE_REQUESTS = 1, 2
MARS_STATIC_SCRATCH_BYTES = 8 << 20
MARS_ERR_SCRATCH = -5


class VerifyOptionsStruct(ctypes.Structure):
    """struct mars_verify_options (a host struct holding device pointers)."""
    _fields_ = [("indicator", ctypes.c_int32), ("n_theta", ctypes.c_int32),
                ("spin_limit", ctypes.c_int32), ("stages", ctypes.c_int32),
                ("out_tokens", ctypes.c_void_p), ("out_len", ctypes.c_void_p),
                ("keep_rows", ctypes.c_void_p), ("keep_offsets", ctypes.c_void_p)]

_lib = None


class MarsError(RuntimeError):
    pass


def lib():
    """Load libmars.so (built by ``paper_2601_15498_amd.build``); fails loudly when missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise MarsError(f"{LIB_PATH} is missing: build it with `python -m paper_2601_15498_amd.build` "
                            "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        L.mars_version.restype = ctypes.c_int
        L.mars_status_string.restype = ctypes.c_char_p
        L.mars_status_string.argtypes = [ctypes.c_int]
        L.mars_workspace_bytes.restype = ctypes.c_size_t
        L.mars_workspace_bytes.argtypes = [ctypes.c_int] * 3
        L.mars_row_reduce.restype = ctypes.c_int
        L.mars_row_reduce.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_int, ctypes.c_int,
                                      ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.mars_row_stats.restype = ctypes.c_int
        L.mars_row_stats.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_float,
                                     ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                     ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.mars_verify.restype = ctypes.c_int
        L.mars_verify.argtypes = ([ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                                   ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_float,
                                   ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int]
                                  + [ctypes.c_void_p] * 8 + [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p])
        L.mars_workspace_bytes_ex.restype = ctypes.c_size_t
        L.mars_workspace_bytes_ex.argtypes = [ctypes.c_int] * 4
        L.mars_verify_ex.restype = ctypes.c_int
        L.mars_verify_ex.argtypes = L.mars_verify.argtypes + [ctypes.POINTER(VerifyOptionsStruct)]
        L.mars_verify_static.restype = ctypes.c_int
        L.mars_verify_static.argtypes = (L.mars_verify.argtypes[:20] + [ctypes.c_void_p,
                                                                        ctypes.POINTER(VerifyOptionsStruct)])
        L.mars_margin_stats.restype = ctypes.c_int
        L.mars_margin_stats.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_float,
                                        ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                        ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_int32),
                                        ctypes.c_void_p, ctypes.c_void_p,
                                        ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.mars_lmhead_workspace_bytes.restype = ctypes.c_size_t
        L.mars_lmhead_workspace_bytes.argtypes = [ctypes.c_int] * 5
        L.mars_lmhead_verify.restype = ctypes.c_int
        L.mars_lmhead_verify.argtypes = ([ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p,
                                          ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int]
                                         + [ctypes.c_void_p] * 7
                                         + [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p,
                                            ctypes.POINTER(VerifyOptionsStruct)])
        L.mars_lmhead_verify_sampling.restype = ctypes.c_int
        L.mars_lmhead_verify_sampling.argtypes = (
            [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
             ctypes.c_int, ctypes.c_void_p, ctypes.c_float, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
             ctypes.c_void_p] + [ctypes.c_void_p] * 8
            + [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.POINTER(VerifyOptionsStruct)])
        _lib = L
    return _lib


def _check(rc: int):
    if rc != MARS_OK:
        raise MarsError(f"mars call failed: {rc} ({lib().mars_status_string(rc).decode()})")


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return MARS_F32
    if t.dtype in (torch.bfloat16, torch.uint16, torch.int16):
        return MARS_BF16
    raise TypeError(f"unsupported element type {t.dtype}")


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


# struct mars_row_stat {float z1; int32 id1; float z2; int32 id2; float sum_exp; int32 relax_ok;}  (24 bytes)
ROW_STAT_WORDS = 6
# struct mars_req_diag {float bonus_prob; float last_residual_norm; int32 residual_passes; int32 last_node;}
REQ_DIAG_WORDS = 4


def mars_version() -> int:
    return int(lib().mars_version())


def mars_workspace_bytes(B: int, N: int, V: int) -> int:
    return int(lib().mars_workspace_bytes(B, N, V))


def mars_workspace_bytes_ex(B: int, N: int, V: int, n_theta: int) -> int:
    return int(lib().mars_workspace_bytes_ex(B, N, V, n_theta))


def alloc_workspace(B: int, N: int, V: int, device="cuda", n_theta: int = 1) -> torch.Tensor:
    n = mars_workspace_bytes_ex(B, N, V, n_theta)
    if n == 0:
        raise MarsError(f"sizes out of range: B={B} N={N} V={V} n_theta={n_theta}")
    return torch.empty(n, dtype=torch.uint8, device=device)


def mars_row_reduce(logits: torch.Tensor, temperature: float, workspace: torch.Tensor) -> None:
    """First stage only (the streaming row reduction); partial results stay in the workspace."""
    B, N, V = logits.shape
    assert logits.is_contiguous()
    _check(lib().mars_row_reduce(_ptr(logits), _dtype_code(logits), float(temperature), B, N, V,
                                 _ptr(workspace), workspace.numel(), _stream()))


def mars_row_stats(logits: torch.Tensor, theta: torch.Tensor, temperature: float, stats: torch.Tensor = None,
                   workspace: torch.Tensor = None) -> torch.Tensor:
    """Row statistics table as an int32 tensor [B*N, 6] (see ``unpack_stats``)."""
    B, N, V = logits.shape
    assert logits.is_contiguous() and theta.dtype == torch.float32 and theta.numel() == B
    if stats is None:
        stats = torch.empty((B * N, ROW_STAT_WORDS), dtype=torch.int32, device=logits.device)
    if workspace is None:
        workspace = alloc_workspace(B, N, V, logits.device)
    _check(lib().mars_row_stats(_ptr(logits), _dtype_code(logits), _ptr(theta), float(temperature), B, N, V,
                                _ptr(stats), _ptr(workspace), workspace.numel(), _stream()))
    return stats


def unpack_stats(stats: torch.Tensor) -> dict:
    s = stats.view(-1, ROW_STAT_WORDS)
    return {"z1": s[:, 0].view(torch.float32), "id1": s[:, 1], "z2": s[:, 2].view(torch.float32),
            "id2": s[:, 3], "sum_exp": s[:, 4].view(torch.float32), "relax_ok": s[:, 5]}


def unpack_diag(diag: torch.Tensor) -> dict:
    d = diag.view(-1, REQ_DIAG_WORDS)
    return {"bonus_prob": d[:, 0].view(torch.float32), "last_residual_norm": d[:, 1].view(torch.float32),
            "residual_passes": d[:, 2], "last_node": d[:, 3]}


class VerifyOutputs:
    """Device tensors written by ``mars_verify`` / ``mars_verify_ex``.  With n_theta = K > 1 every tensor
    has a leading axis of length K; with want_commit the committed sequence and kept cache rows too."""

    def __init__(self, B: int, N: int, device, want_stats: bool = True, want_diag: bool = True,
                 n_theta: int = 1, want_commit: bool = False):
        lead = (n_theta,) if n_theta > 1 else ()
        self.n_theta = n_theta
        self.accept_mask = torch.empty(lead + (B, N), dtype=torch.uint8, device=device)
        self.accept_len = torch.empty(lead + (B,), dtype=torch.int32, device=device)
        self.path_idx = torch.empty(lead + (B, N), dtype=torch.int32, device=device)
        self.bonus_token = torch.empty(lead + (B,), dtype=torch.int32, device=device)
        self.decision = torch.empty(lead + (B, N), dtype=torch.uint8, device=device)
        self.request_status = torch.empty(lead + (B,), dtype=torch.int32, device=device)
        self.stats = (torch.empty(lead + (B * N, ROW_STAT_WORDS), dtype=torch.int32, device=device)
                      if want_stats else None)
        self.diag = torch.empty(lead + (B, REQ_DIAG_WORDS), dtype=torch.int32, device=device) if want_diag else None
        self.out_tokens = self.out_len = self.keep_rows = self.keep_offsets = None
        if want_commit:
            self.out_tokens = torch.empty(lead + (B, N), dtype=torch.int32, device=device)
            self.out_len = torch.empty(lead + (B,), dtype=torch.int32, device=device)
            self.keep_rows = torch.empty(lead + (B * N,), dtype=torch.int32, device=device)
            self.keep_offsets = torch.empty(lead + (B + 1,), dtype=torch.int32, device=device)


def mars_verify(logits: torch.Tensor, draft_tokens: torch.Tensor, tree_parent: torch.Tensor,
                theta: torch.Tensor, temperature: float, uniforms: torch.Tensor = None,
                draft_probs: torch.Tensor = None, out: VerifyOutputs = None,
                workspace: torch.Tensor = None) -> VerifyOutputs:
    """The whole verification pass; see include/mars.h for argument meaning and layout."""
    B, N, V = logits.shape
    dev = logits.device
    assert logits.is_contiguous()
    assert draft_tokens.dtype == torch.int32 and draft_tokens.shape == (B, N) and draft_tokens.is_contiguous()
    assert tree_parent.dtype == torch.int32 and tree_parent.shape == (B, N) and tree_parent.is_contiguous()
    assert theta.dtype == torch.float32 and theta.numel() == B
    if uniforms is not None:
        assert uniforms.dtype == torch.float32 and uniforms.shape == (B, N + 1) and uniforms.is_contiguous()
    dcode = 0
    if draft_probs is not None:
        assert draft_probs.shape == (B, N, V) and draft_probs.is_contiguous()
        dcode = _dtype_code(draft_probs)
    if out is None:
        out = VerifyOutputs(B, N, dev)
    if workspace is None:
        workspace = alloc_workspace(B, N, V, dev)
    _check(lib().mars_verify(_ptr(logits), _dtype_code(logits), _ptr(draft_tokens), _ptr(tree_parent),
                             _ptr(draft_probs), dcode, _ptr(theta), float(temperature), _ptr(uniforms),
                             B, N, V, _ptr(out.accept_mask), _ptr(out.accept_len), _ptr(out.path_idx),
                             _ptr(out.bonus_token), _ptr(out.decision), _ptr(out.request_status),
                             _ptr(out.stats), _ptr(out.diag), _ptr(workspace), workspace.numel(), _stream()))
    return out


def mars_verify_ex(logits: torch.Tensor, draft_tokens: torch.Tensor, tree_parent: torch.Tensor,
                   theta: torch.Tensor, temperature: float, uniforms: torch.Tensor = None,
                   draft_probs: torch.Tensor = None, out: VerifyOutputs = None, workspace: torch.Tensor = None,
                   indicator: int = MARS_IND_LOGIT_RATIO, n_theta: int = 1,
                   want_commit: bool = False, spin_limit: int = 0, stages: int = 0) -> VerifyOutputs:
    """mars_verify with options: low-margin indicator, theta[K,B] swept in one pass, committed sequence and
    kept cache rows.  See include/mars.h."""
    B, N, V = logits.shape
    dev = logits.device
    assert logits.is_contiguous()
    assert draft_tokens.dtype == torch.int32 and draft_tokens.shape == (B, N) and draft_tokens.is_contiguous()
    assert tree_parent.dtype == torch.int32 and tree_parent.shape == (B, N) and tree_parent.is_contiguous()
    assert theta.dtype == torch.float32 and theta.numel() == n_theta * B and theta.is_contiguous()
    if uniforms is not None:
        assert uniforms.dtype == torch.float32 and uniforms.shape == (B, N + 1) and uniforms.is_contiguous()
    dcode = 0
    if draft_probs is not None:
        assert draft_probs.shape == (B, N, V) and draft_probs.is_contiguous()
        dcode = _dtype_code(draft_probs)
    if out is None:
        out = VerifyOutputs(B, N, dev, n_theta=n_theta, want_commit=want_commit)
    assert out.n_theta == n_theta
    if workspace is None:
        workspace = alloc_workspace(B, N, V, dev, n_theta)
    opt = VerifyOptionsStruct(int(indicator), int(n_theta), int(spin_limit), int(stages),
                              None if out.out_tokens is None else out.out_tokens.data_ptr(),
                              None if out.out_len is None else out.out_len.data_ptr(),
                              None if out.keep_rows is None else out.keep_rows.data_ptr(),
                              None if out.keep_offsets is None else out.keep_offsets.data_ptr())
    _check(lib().mars_verify_ex(_ptr(logits), _dtype_code(logits), _ptr(draft_tokens), _ptr(tree_parent),
                                _ptr(draft_probs), dcode, _ptr(theta), float(temperature), _ptr(uniforms),
                                B, N, V, _ptr(out.accept_mask), _ptr(out.accept_len), _ptr(out.path_idx),
                                _ptr(out.bonus_token), _ptr(out.decision), _ptr(out.request_status),
                                _ptr(out.stats), _ptr(out.diag), _ptr(workspace), workspace.numel(), _stream(),
                                ctypes.byref(opt)))
    return out


def mars_verify_static(logits: torch.Tensor, draft_tokens: torch.Tensor, tree_parent: torch.Tensor,
                       theta: torch.Tensor, temperature: float, uniforms: torch.Tensor = None,
                       draft_probs: torch.Tensor = None, out: VerifyOutputs = None,
                       indicator: int = MARS_IND_LOGIT_RATIO, n_theta: int = 1,
                       want_commit: bool = False, spin_limit: int = 0) -> VerifyOutputs:
    """mars_verify_ex on the library's own static scratch array (no workspace argument, nothing allocated by
    the call itself; ``out`` should be given by a caller that must not allocate).  See include/mars.h."""
    B, N, V = logits.shape
    dev = logits.device
    assert logits.is_contiguous()
    assert draft_tokens.dtype == torch.int32 and draft_tokens.shape == (B, N) and draft_tokens.is_contiguous()
    assert tree_parent.dtype == torch.int32 and tree_parent.shape == (B, N) and tree_parent.is_contiguous()
    assert theta.dtype == torch.float32 and theta.numel() == n_theta * B and theta.is_contiguous()
    if uniforms is not None:
        assert uniforms.dtype == torch.float32 and uniforms.shape == (B, N + 1) and uniforms.is_contiguous()
    dcode = 0
    if draft_probs is not None:
        assert draft_probs.shape == (B, N, V) and draft_probs.is_contiguous()
        dcode = _dtype_code(draft_probs)
    if out is None:
        out = VerifyOutputs(B, N, dev, n_theta=n_theta, want_commit=want_commit)
    assert out.n_theta == n_theta
    opt = VerifyOptionsStruct(int(indicator), int(n_theta), int(spin_limit), 0,
                              None if out.out_tokens is None else out.out_tokens.data_ptr(),
                              None if out.out_len is None else out.out_len.data_ptr(),
                              None if out.keep_rows is None else out.keep_rows.data_ptr(),
                              None if out.keep_offsets is None else out.keep_offsets.data_ptr())
    _check(lib().mars_verify_static(_ptr(logits), _dtype_code(logits), _ptr(draft_tokens), _ptr(tree_parent),
                                    _ptr(draft_probs), dcode, _ptr(theta), float(temperature), _ptr(uniforms),
                                    B, N, V, _ptr(out.accept_mask), _ptr(out.accept_len), _ptr(out.path_idx),
                                    _ptr(out.bonus_token), _ptr(out.decision), _ptr(out.request_status),
                                    _ptr(out.stats), _ptr(out.diag), _stream(), ctypes.byref(opt)))
    return out


# struct mars_margin_row {float z1; float z2; float ratio; float prob_ratio;}
MARGIN_ROW_WORDS = 4


def margin_counts_len(bins) -> int:
    return sum(int(b) + 2 for b in bins) + 4


def mars_margin_stats(logits: torch.Tensor, theta: torch.Tensor, temperature: float, ranges, bins,
                      rows_out: torch.Tensor = None, counts: torch.Tensor = None, workspace: torch.Tensor = None,
                      want_rows: bool = True):
    """Top-2 statistics per row ([B*N, 4] fp32: z1, z2, z2/z1, p2/p1) and their histograms (one uint32 tensor:
    three histograms of bins+2 counters each, then rows, z1 < 0, z1 <= 0, low-margin rows).  ranges: six floats
    (lo, hi of z1, of z2/z1, of p2/p1); bins: three ints.  See include/mars.h."""
    B, N, V = logits.shape
    dev = logits.device
    assert logits.is_contiguous() and theta.dtype == torch.float32 and theta.numel() == B
    rg = (ctypes.c_float * 6)(*[float(x) for x in ranges])
    bn = (ctypes.c_int32 * 3)(*[int(x) for x in bins])
    if rows_out is None and want_rows:
        rows_out = torch.empty((B * N, MARGIN_ROW_WORDS), dtype=torch.float32, device=dev)
    if counts is None:
        counts = torch.empty((margin_counts_len(bins),), dtype=torch.int32, device=dev)
    if workspace is None:
        workspace = alloc_workspace(B, N, V, dev)
    _check(lib().mars_margin_stats(_ptr(logits), _dtype_code(logits), _ptr(theta), float(temperature), B, N, V,
                                   rg, bn, _ptr(rows_out), _ptr(counts), _ptr(workspace), workspace.numel(),
                                   _stream()))
    return rows_out, counts


def mars_lmhead_workspace_bytes(B: int, N: int, V: int, H: int, n_theta: int = 1) -> int:
    return int(lib().mars_lmhead_workspace_bytes(B, N, V, H, n_theta))


def mars_lmhead_verify(hidden: torch.Tensor, weight: torch.Tensor, draft_tokens: torch.Tensor,
                       tree_parent: torch.Tensor, theta: torch.Tensor, out: VerifyOutputs = None,
                       workspace: torch.Tensor = None, indicator: int = MARS_IND_LOGIT_RATIO, n_theta: int = 1,
                       want_commit: bool = False, stages: int = 0) -> VerifyOutputs:
    """Greedy verification from the last hidden states [B,N,H] and the LM-head weight [V,H] (both bf16, or
    their bit patterns): the logits are formed, reduced and dropped inside one kernel.  See include/mars.h."""
    B, N, H = hidden.shape
    V = weight.shape[0]
    dev = hidden.device
    assert hidden.is_contiguous() and weight.is_contiguous() and weight.shape == (V, H)
    assert _dtype_code(hidden) == MARS_BF16 and _dtype_code(weight) == MARS_BF16
    assert draft_tokens.dtype == torch.int32 and draft_tokens.shape == (B, N) and draft_tokens.is_contiguous()
    assert tree_parent.dtype == torch.int32 and tree_parent.shape == (B, N) and tree_parent.is_contiguous()
    assert theta.dtype == torch.float32 and theta.numel() == n_theta * B and theta.is_contiguous()
    if out is None:
        out = VerifyOutputs(B, N, dev, want_diag=False, n_theta=n_theta, want_commit=want_commit)
    assert out.n_theta == n_theta
    if workspace is None:
        n = mars_lmhead_workspace_bytes(B, N, V, H, n_theta)
        if n == 0:
            raise MarsError(f"sizes out of range: B={B} N={N} V={V} H={H} n_theta={n_theta}")
        workspace = torch.empty(n, dtype=torch.uint8, device=dev)
    opt = VerifyOptionsStruct(int(indicator), int(n_theta), 0, int(stages),
                              None if out.out_tokens is None else out.out_tokens.data_ptr(),
                              None if out.out_len is None else out.out_len.data_ptr(),
                              None if out.keep_rows is None else out.keep_rows.data_ptr(),
                              None if out.keep_offsets is None else out.keep_offsets.data_ptr())
    _check(lib().mars_lmhead_verify(_ptr(hidden), _ptr(weight), H, _ptr(draft_tokens), _ptr(tree_parent), _ptr(theta),
                                    B, N, V, _ptr(out.accept_mask), _ptr(out.accept_len), _ptr(out.path_idx),
                                    _ptr(out.bonus_token), _ptr(out.decision), _ptr(out.request_status),
                                    _ptr(out.stats), _ptr(workspace), workspace.numel(), _stream(),
                                    ctypes.byref(opt)))
    return out


def mars_lmhead_verify_sampling(hidden: torch.Tensor, weight: torch.Tensor, draft_tokens: torch.Tensor,
                                tree_parent: torch.Tensor, theta: torch.Tensor, temperature: float,
                                uniforms: torch.Tensor, draft_probs: torch.Tensor = None,
                                logits_out: torch.Tensor = None, out: VerifyOutputs = None,
                                workspace: torch.Tensor = None, indicator: int = MARS_IND_LOGIT_RATIO,
                                n_theta: int = 1, want_commit: bool = False, spin_limit: int = 0, stages: int = 0):
    """Sampling-mode verification from the last hidden states [B,N,H] and the LM-head weight [V,H] (both bf16, or
    their bit patterns): one kernel forms the logits, writes them to ``logits_out`` [B,N,V] (bf16 bit patterns) and
    takes each row's top-2 and sum of exponentials on the way; the sampling walk follows.  Returns
    (outputs, logits_out).  See include/mars.h."""
    B, N, H = hidden.shape
    V = weight.shape[0]
    dev = hidden.device
    assert hidden.is_contiguous() and weight.is_contiguous() and weight.shape == (V, H)
    assert _dtype_code(hidden) == MARS_BF16 and _dtype_code(weight) == MARS_BF16
    assert draft_tokens.dtype == torch.int32 and draft_tokens.shape == (B, N) and draft_tokens.is_contiguous()
    assert tree_parent.dtype == torch.int32 and tree_parent.shape == (B, N) and tree_parent.is_contiguous()
    assert theta.dtype == torch.float32 and theta.numel() == n_theta * B and theta.is_contiguous()
    assert uniforms.dtype == torch.float32 and uniforms.shape == (B, N + 1) and uniforms.is_contiguous()
    dcode = 0
    if draft_probs is not None:
        assert draft_probs.shape == (B, N, V) and draft_probs.is_contiguous()
        dcode = _dtype_code(draft_probs)
    if logits_out is None:
        logits_out = torch.empty((B, N, V), dtype=torch.uint16, device=dev)
    assert logits_out.shape == (B, N, V) and logits_out.is_contiguous() and _dtype_code(logits_out) == MARS_BF16
    if out is None:
        out = VerifyOutputs(B, N, dev, want_diag=True, n_theta=n_theta, want_commit=want_commit)
    assert out.n_theta == n_theta
    if workspace is None:
        n = mars_lmhead_workspace_bytes(B, N, V, H, n_theta)
        if n == 0:
            raise MarsError(f"sizes out of range: B={B} N={N} V={V} H={H} n_theta={n_theta}")
        workspace = torch.empty(n, dtype=torch.uint8, device=dev)
    opt = VerifyOptionsStruct(int(indicator), int(n_theta), int(spin_limit), int(stages),
                              None if out.out_tokens is None else out.out_tokens.data_ptr(),
                              None if out.out_len is None else out.out_len.data_ptr(),
                              None if out.keep_rows is None else out.keep_rows.data_ptr(),
                              None if out.keep_offsets is None else out.keep_offsets.data_ptr())
    _check(lib().mars_lmhead_verify_sampling(
        _ptr(hidden), _ptr(weight), H, _ptr(draft_tokens), _ptr(tree_parent), _ptr(draft_probs), dcode, _ptr(theta),
        float(temperature), _ptr(uniforms), B, N, V, _ptr(logits_out), _ptr(out.accept_mask), _ptr(out.accept_len),
        _ptr(out.path_idx), _ptr(out.bonus_token), _ptr(out.decision), _ptr(out.request_status), _ptr(out.stats),
        _ptr(out.diag), _ptr(workspace), workspace.numel(), _stream(), ctypes.byref(opt)))
    return out, logits_out
