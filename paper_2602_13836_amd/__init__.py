"""Python binding of libspecvocab.so (the C ABI declared in include/specvocab.h).

Argument marshalling only: every step of the draft-step path runs in the HIP kernels of the
library.  torch is used for device memory and the current stream, nothing else.  There is no
CPU fallback: if the library has not been built, or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspecvocab.so")

SV_OK = 0
SV_F32, SV_BF16 = 0, 1
SV_IDX_PER_ROW, SV_IDX_PER_STEP = 0, 1
SV_OP_SELECT, SV_OP_SUBSET_LOGITS, SV_OP_DRAFT_TOPK, SV_OP_DENSE_LOGITS, SV_OP_DRAFT_STEP = 0, 1, 2, 3, 4
SV_OP_INDEXED_HEAD_NAIVE = 5
SV_OP_AUX_LOG_SOFTMAX = 6
SV_IDX_PADDED = 4        # OR into idx_mode: the list may hold padding slots (-1)
SV_IDX_SORTED = 8        # OR into idx_mode: every list is sorted by ascending id (what select emits)
MAX_KD = 64
SELECT_SAMPLE = 8192     # sampled tokens of the batch selection: ids floor(j * V / SELECT_SAMPLE)

EXPORTS = (
    "specvocab_version",
    "specvocab_init",
    "specvocab_status_string",
    "specvocab_workspace_bytes",
    "specvocab_select",
    "specvocab_select_static",
    "specvocab_select_threshold",
    "specvocab_subset_logits",
    "specvocab_draft_topk",
    "specvocab_draft_step",
    "specvocab_indexed_head_naive",
    "specvocab_pack_rows",
    "specvocab_aux_log_softmax",
    "specvocab_stream_read_probe",
    "specvocab_dense_logits",
)


class SpecVocabError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({status_string(status)})")


_lib = None


def load_library(path: Optional[str] = None) -> ctypes.CDLL:
    """Load the built library (never builds it). Raises if it is missing."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise FileNotFoundError(
            f"{p} not found: build it first (python -m paper_2602_13836_amd.build, or "
            f"__graft_entry__.build()); there is no fallback path")
    lib = ctypes.CDLL(p)
    i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
    lib.specvocab_version.restype = ci
    lib.specvocab_version.argtypes = []
    lib.specvocab_status_string.restype = ctypes.c_char_p
    lib.specvocab_status_string.argtypes = [ci]
    lib.specvocab_workspace_bytes.restype = ci
    lib.specvocab_workspace_bytes.argtypes = [ci, i64, i64, i64, i64, i64, i64, ci, ci,
                                              ctypes.POINTER(ctypes.c_size_t)]
    lib.specvocab_select.restype = ci
    lib.specvocab_select.argtypes = [vp, i64, i64, i64, vp, i64, vp, i64, ci, i64, vp, vp, vp,
                                     ctypes.c_size_t, vp]
    lib.specvocab_init.restype = ci
    lib.specvocab_init.argtypes = []
    lib.specvocab_select_static.restype = ci
    lib.specvocab_select_static.argtypes = [vp, i64, i64, i64, vp, i64, vp, i64, ci, i64, vp, vp, vp]
    lib.specvocab_select_threshold.restype = ci
    lib.specvocab_select_threshold.argtypes = [vp, i64, i64, i64, vp, i64, vp, i64, ci, i64, ctypes.c_float, vp, vp,
                                               vp, ctypes.c_size_t, vp]
    lib.specvocab_subset_logits.restype = ci
    lib.specvocab_subset_logits.argtypes = [vp, i64, i64, i64, vp, i64, i64, ci, vp, i64, ci, vp, vp,
                                            ctypes.c_size_t, vp]
    lib.specvocab_indexed_head_naive.restype = ci
    lib.specvocab_indexed_head_naive.argtypes = lib.specvocab_subset_logits.argtypes
    lib.specvocab_aux_log_softmax.restype = ci
    lib.specvocab_aux_log_softmax.argtypes = [vp, i64, i64, i64, vp, i64, vp, i64, ci, vp, vp, ctypes.c_size_t, vp]
    lib.specvocab_pack_rows.restype = ci
    lib.specvocab_pack_rows.argtypes = [vp, i64, i64, i64, ci, vp, i64, vp, vp]
    lib.specvocab_draft_topk.restype = ci
    lib.specvocab_draft_topk.argtypes = [vp, vp, ci, i64, i64, i64, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.specvocab_draft_step.restype = ci
    lib.specvocab_draft_step.argtypes = [vp, i64, i64, i64, vp, i64, i64, ci, vp, i64, ci, i64, vp, vp, vp, vp, vp,
                                         ctypes.c_size_t, vp]
    lib.specvocab_stream_read_probe.restype = ci
    lib.specvocab_stream_read_probe.argtypes = [vp, ctypes.c_size_t, vp, ctypes.c_size_t, vp]
    lib.specvocab_dense_logits.restype = ci
    lib.specvocab_dense_logits.argtypes = [vp, i64, i64, i64, vp, i64, i64, ci, vp, vp, ctypes.c_size_t, vp]
    if path is None:
        _lib = lib
    return lib


STATIC_SCRATCH_BYTES = 8 << 20       # SPECVOCAB_STATIC_SCRATCH_BYTES


def init() -> None:
    """specvocab_init: one-time set-up of the current device (needed explicitly only before a first call that
    would fall inside a stream capture)."""
    _check(load_library().specvocab_init(), "specvocab_init")


def version() -> int:
    return int(load_library().specvocab_version())


def status_string(status: int) -> str:
    return load_library().specvocab_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != SV_OK:
        raise SpecVocabError(status, where)


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return SV_F32
    if t.dtype == torch.bfloat16:
        return SV_BF16
    raise TypeError(f"storage dtype must be float32 or bfloat16, got {t.dtype}")


def _mat(t: torch.Tensor, name: str) -> Tuple[int, int, int]:
    """(rows, cols, row stride in elements) of a device matrix with contiguous rows."""
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if t.dim() != 2 or t.stride(1) != 1:
        raise ValueError(f"{name} must be a 2-D tensor with contiguous rows")
    ld = t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1])
    return t.shape[0], t.shape[1], ld


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream: Optional[torch.cuda.Stream]):
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def _idx(idx: torch.Tensor, rows: int) -> Tuple[int, int]:
    if not idx.is_cuda or idx.dtype != torch.int32 or not idx.is_contiguous():
        raise ValueError("idx must be a contiguous int32 GPU tensor")
    if idx.dim() == 1:
        return SV_IDX_PER_STEP, idx.shape[0]
    if idx.dim() == 2 and idx.shape[0] == rows:
        return SV_IDX_PER_ROW, idx.shape[1]
    raise ValueError("idx must be [k] (one set per step) or [rows x k]")


def workspace_bytes(op: int, rows: int = 0, d: int = 0, V: int = 0, k: int = 0, d_prime: int = 0,
                    kd: int = 0, dt: int = SV_BF16, idx_mode: int = SV_IDX_PER_ROW) -> int:
    out = ctypes.c_size_t(0)
    _check(load_library().specvocab_workspace_bytes(op, rows, d, V, k, d_prime, kd, dt, idx_mode,
                                                    ctypes.byref(out)), "specvocab_workspace_bytes")
    return int(out.value)


def _workspace(nbytes: int, device, ws: Optional[torch.Tensor]) -> Optional[torch.Tensor]:
    if ws is not None:
        if ws.dtype != torch.uint8 or not ws.is_contiguous() or ws.numel() < nbytes:
            raise ValueError(f"workspace must be a contiguous uint8 tensor of >= {nbytes} bytes")
        return ws
    if nbytes == 0:
        return None
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def select(h: torch.Tensor, W_down: torch.Tensor, W_vocab: torch.Tensor, k: int,
           idx_out: Optional[torch.Tensor] = None, scores_out: Optional[torch.Tensor] = None,
           want_scores: bool = False, ws: Optional[torch.Tensor] = None,
           stream: Optional[torch.cuda.Stream] = None, tau: Optional[float] = None):
    """specvocab_select: ids of the k largest approximate logits per row, ascending.
    Returns (idx [rows x k] int32, scores [rows x k] float32 or None).
    tau: specvocab_select_threshold -- selected tokens scoring below tau become padding slots (-1)."""
    rows, d, ldh = _mat(h, "h")
    dp, d2, ldd = _mat(W_down, "W_down")
    V, dp2, ldv = _mat(W_vocab, "W_vocab")
    if d2 != d or dp2 != dp or ldd != d or ldv != dp:
        raise ValueError("W_down must be a dense [d' x d] and W_vocab a dense [V x d']")
    dt = _dt(h)
    if _dt(W_down) != dt or _dt(W_vocab) != dt:
        raise TypeError("h, W_down and W_vocab must share a dtype")
    if idx_out is None:
        idx_out = torch.empty((rows, k), dtype=torch.int32, device=h.device)
    if scores_out is None and want_scores:
        scores_out = torch.empty((rows, k), dtype=torch.float32, device=h.device)
    nbytes = workspace_bytes(SV_OP_SELECT, rows, d, V, k, dp, 0, dt)
    ws = _workspace(nbytes, h.device, ws)
    if tau is None:
        _check(load_library().specvocab_select(_ptr(h), rows, d, ldh, _ptr(W_down), dp, _ptr(W_vocab), V, dt, k,
                                               _ptr(idx_out), _ptr(scores_out), _ptr(ws),
                                               0 if ws is None else ws.numel(), _stream(stream)),
               "specvocab_select")
    else:
        _check(load_library().specvocab_select_threshold(_ptr(h), rows, d, ldh, _ptr(W_down), dp, _ptr(W_vocab), V,
                                                         dt, k, ctypes.c_float(tau), _ptr(idx_out),
                                                         _ptr(scores_out), _ptr(ws),
                                                         0 if ws is None else ws.numel(), _stream(stream)),
               "specvocab_select_threshold")
    return idx_out, scores_out


def select_static(h: torch.Tensor, W_down: torch.Tensor, W_vocab: torch.Tensor, k: int,
                  idx_out: torch.Tensor, scores_out: Optional[torch.Tensor] = None,
                  stream: Optional[torch.cuda.Stream] = None):
    """specvocab_select_static: specvocab_select on the library's static device scratch.  Allocates nothing:
    the caller passes the outputs."""
    rows, d, ldh = _mat(h, "h")
    dp, d2, ldd = _mat(W_down, "W_down")
    V, dp2, ldv = _mat(W_vocab, "W_vocab")
    if d2 != d or dp2 != dp or ldd != d or ldv != dp:
        raise ValueError("W_down must be a dense [d' x d] and W_vocab a dense [V x d']")
    dt = _dt(h)
    if _dt(W_down) != dt or _dt(W_vocab) != dt:
        raise TypeError("h, W_down and W_vocab must share a dtype")
    if idx_out.shape != (rows, k) or idx_out.dtype != torch.int32 or not idx_out.is_contiguous():
        raise ValueError("idx_out must be a contiguous [rows x k] int32 GPU tensor")
    _check(load_library().specvocab_select_static(_ptr(h), rows, d, ldh, _ptr(W_down), dp, _ptr(W_vocab), V, dt, k,
                                                  _ptr(idx_out), _ptr(scores_out), _stream(stream)),
           "specvocab_select_static")
    return idx_out, scores_out


def subset_logits(h: torch.Tensor, U: torch.Tensor, idx: torch.Tensor,
                  out: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None,
                  stream: Optional[torch.cuda.Stream] = None, padded: bool = False,
                  sorted_lists: bool = False) -> torch.Tensor:
    """specvocab_subset_logits: out[r, j] = <U[idx(r, j)], h_r>, [rows x k] float32.
    padded=True: idx may hold padding slots (-1), whose logit is -inf.
    sorted_lists=True: the caller declares every list sorted by ascending id (SV_IDX_SORTED)."""
    rows, d, ldh = _mat(h, "h")
    V, d2, ldu = _mat(U, "U")
    if d2 != d:
        raise ValueError("U and h disagree on d")
    dt = _dt(h)
    if _dt(U) != dt:
        raise TypeError("h and U must share a dtype")
    mode, k = _idx(idx, rows)
    if padded:
        mode |= SV_IDX_PADDED
    if sorted_lists:
        mode |= SV_IDX_SORTED
    if out is None:
        out = torch.empty((rows, k), dtype=torch.float32, device=h.device)
    nbytes = workspace_bytes(SV_OP_SUBSET_LOGITS, rows, d, V, k, 0, 0, dt, mode)
    ws = _workspace(nbytes, h.device, ws)
    _check(load_library().specvocab_subset_logits(_ptr(h), rows, d, ldh, _ptr(U), V, ldu, dt, _ptr(idx), k,
                                                  mode, _ptr(out), _ptr(ws),
                                                  0 if ws is None else ws.numel(), _stream(stream)),
           "specvocab_subset_logits")
    return out


def indexed_head_naive(h: torch.Tensor, U: torch.Tensor, idx: torch.Tensor,
                       out: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None,
                       stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """specvocab_indexed_head_naive: the comparator that materialises U[idx] and multiplies the copy."""
    rows, d, ldh = _mat(h, "h")
    V, d2, ldu = _mat(U, "U")
    if d2 != d:
        raise ValueError("U and h disagree on d")
    dt = _dt(h)
    if _dt(U) != dt:
        raise TypeError("h and U must share a dtype")
    mode, k = _idx(idx, rows)
    if out is None:
        out = torch.empty((rows, k), dtype=torch.float32, device=h.device)
    nbytes = workspace_bytes(SV_OP_INDEXED_HEAD_NAIVE, rows, d, V, k, 0, 0, dt, mode)
    ws = _workspace(nbytes, h.device, ws)
    _check(load_library().specvocab_indexed_head_naive(_ptr(h), rows, d, ldh, _ptr(U), V, ldu, dt, _ptr(idx), k,
                                                       mode, _ptr(out), _ptr(ws),
                                                       0 if ws is None else ws.numel(), _stream(stream)),
           "specvocab_indexed_head_naive")
    return out


def aux_log_softmax(h: torch.Tensor, W_down: torch.Tensor, W_vocab: torch.Tensor,
                    out: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None,
                    stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """specvocab_aux_log_softmax: log q_aux = log softmax(W_vocab (W_down h)) over the whole vocabulary,
    [rows x V] float32."""
    rows, d, ldh = _mat(h, "h")
    dp, d2, ldd = _mat(W_down, "W_down")
    V, dp2, ldv = _mat(W_vocab, "W_vocab")
    if d2 != d or dp2 != dp or ldd != d or ldv != dp:
        raise ValueError("W_down must be a dense [d' x d] and W_vocab a dense [V x d']")
    dt = _dt(h)
    if _dt(W_down) != dt or _dt(W_vocab) != dt:
        raise TypeError("h, W_down and W_vocab must share a dtype")
    if out is None:
        out = torch.empty((rows, V), dtype=torch.float32, device=h.device)
    elif out.shape != (rows, V) or out.dtype != torch.float32 or not out.is_contiguous() or not out.is_cuda:
        raise ValueError("out must be a contiguous [rows x V] float32 GPU tensor")
    nbytes = workspace_bytes(SV_OP_AUX_LOG_SOFTMAX, rows, d, V, 0, dp, 0, dt)
    ws = _workspace(nbytes, h.device, ws)
    _check(load_library().specvocab_aux_log_softmax(_ptr(h), rows, d, ldh, _ptr(W_down), dp, _ptr(W_vocab), V, dt,
                                                    _ptr(out), _ptr(ws), 0 if ws is None else ws.numel(),
                                                    _stream(stream)),
           "specvocab_aux_log_softmax")
    return out


def pack_rows(U: torch.Tensor, idx: torch.Tensor, out: Optional[torch.Tensor] = None,
              stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """specvocab_pack_rows: U' = U[idx, :] as a dense [k x d] matrix (static-vocabulary mode)."""
    V, d, ldu = _mat(U, "U")
    dt = _dt(U)
    if not idx.is_cuda or idx.dtype != torch.int32 or idx.dim() != 1 or not idx.is_contiguous():
        raise ValueError("idx must be a contiguous [k] int32 GPU tensor")
    k = idx.shape[0]
    if out is None:
        out = torch.empty((k, d), dtype=U.dtype, device=U.device)
    elif out.shape != (k, d) or out.dtype != U.dtype or not out.is_contiguous() or not out.is_cuda:
        raise ValueError("out must be a contiguous [k x d] GPU tensor of U's dtype")
    _check(load_library().specvocab_pack_rows(_ptr(U), V, d, ldu, dt, _ptr(idx), k, _ptr(out), _stream(stream)),
           "specvocab_pack_rows")
    return out


def draft_topk(logits: torch.Tensor, idx: torch.Tensor, kd: int,
               tok_out: Optional[torch.Tensor] = None, prob_out: Optional[torch.Tensor] = None,
               probs_full_out: Optional[torch.Tensor] = None, want_probs: bool = False,
               ws: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None):
    """specvocab_draft_topk: subset softmax + top-kd tokens per row.
    Returns (tok [rows x kd] int32, prob [rows x kd] float32, q_K [rows x k] float32 or None)."""
    if not logits.is_cuda or logits.dtype != torch.float32 or logits.dim() != 2 or not logits.is_contiguous():
        raise ValueError("logits must be a contiguous [rows x k] float32 GPU tensor")
    rows, k = logits.shape
    mode, k2 = _idx(idx, rows)
    if k2 != k:
        raise ValueError("idx and logits disagree on k")
    if tok_out is None:
        tok_out = torch.empty((rows, kd), dtype=torch.int32, device=logits.device)
    if prob_out is None:
        prob_out = torch.empty((rows, kd), dtype=torch.float32, device=logits.device)
    if probs_full_out is None and want_probs:
        probs_full_out = torch.empty((rows, k), dtype=torch.float32, device=logits.device)
    nbytes = workspace_bytes(SV_OP_DRAFT_TOPK, rows, 0, 0, k, 0, kd, SV_F32, mode)
    ws = _workspace(nbytes, logits.device, ws)
    _check(load_library().specvocab_draft_topk(_ptr(logits), _ptr(idx), mode, rows, k, kd, _ptr(tok_out),
                                               _ptr(prob_out), _ptr(probs_full_out), _ptr(ws),
                                               0 if ws is None else ws.numel(), _stream(stream)),
           "specvocab_draft_topk")
    return tok_out, prob_out, probs_full_out


def draft_step(h: torch.Tensor, U: torch.Tensor, idx: torch.Tensor, kd: int,
               logits_out: Optional[torch.Tensor] = None, tok_out: Optional[torch.Tensor] = None,
               prob_out: Optional[torch.Tensor] = None, probs_full_out: Optional[torch.Tensor] = None,
               want_probs: bool = False, ws: Optional[torch.Tensor] = None,
               stream: Optional[torch.cuda.Stream] = None, padded: bool = False, sorted_lists: bool = False):
    """specvocab_draft_step: subset logits, then subset softmax and top-kd tokens of every row,
    enqueued back to back. Returns (logits [rows x k], tok [rows x kd], prob [rows x kd],
    q_K [rows x k] or None)."""
    rows, d, ldh = _mat(h, "h")
    V, d2, ldu = _mat(U, "U")
    if d2 != d:
        raise ValueError("U and h disagree on d")
    dt = _dt(h)
    if _dt(U) != dt:
        raise TypeError("h and U must share a dtype")
    mode, k = _idx(idx, rows)
    if padded:
        mode |= SV_IDX_PADDED
    if sorted_lists:
        mode |= SV_IDX_SORTED
    dev = h.device
    if logits_out is None:
        logits_out = torch.empty((rows, k), dtype=torch.float32, device=dev)
    if tok_out is None:
        tok_out = torch.empty((rows, kd), dtype=torch.int32, device=dev)
    if prob_out is None:
        prob_out = torch.empty((rows, kd), dtype=torch.float32, device=dev)
    if probs_full_out is None and want_probs:
        probs_full_out = torch.empty((rows, k), dtype=torch.float32, device=dev)
    nbytes = workspace_bytes(SV_OP_DRAFT_STEP, rows, d, V, k, 0, kd, dt, mode)
    ws = _workspace(nbytes, dev, ws)
    _check(load_library().specvocab_draft_step(_ptr(h), rows, d, ldh, _ptr(U), V, ldu, dt, _ptr(idx), k, mode, kd,
                                               _ptr(logits_out), _ptr(tok_out), _ptr(prob_out),
                                               _ptr(probs_full_out), _ptr(ws), 0 if ws is None else ws.numel(),
                                               _stream(stream)),
           "specvocab_draft_step")
    return logits_out, tok_out, prob_out, probs_full_out


def stream_read_probe(buf: torch.Tensor, ws: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> None:
    """specvocab_stream_read_probe: one plain streaming read of buf (measurement aid)."""
    if not buf.is_cuda or not buf.is_contiguous() or not ws.is_cuda or ws.dtype != torch.uint8:
        raise ValueError("buf and ws must be contiguous GPU tensors (ws uint8)")
    nbytes = buf.numel() * buf.element_size()
    _check(load_library().specvocab_stream_read_probe(_ptr(buf), nbytes - nbytes % 16, _ptr(ws), ws.numel(),
                                                      _stream(stream)), "specvocab_stream_read_probe")


def dense_logits(h: torch.Tensor, U: torch.Tensor, out: Optional[torch.Tensor] = None,
                 ws: Optional[torch.Tensor] = None,
                 stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """specvocab_dense_logits: the full-vocabulary baseline, out[r, v] = <U[v], h_r>."""
    rows, d, ldh = _mat(h, "h")
    V, d2, ldu = _mat(U, "U")
    if d2 != d:
        raise ValueError("U and h disagree on d")
    dt = _dt(h)
    if _dt(U) != dt:
        raise TypeError("h and U must share a dtype")
    if out is None:
        out = torch.empty((rows, V), dtype=torch.float32, device=h.device)
    nbytes = workspace_bytes(SV_OP_DENSE_LOGITS, rows, d, V, 0, 0, 0, dt)
    ws = _workspace(nbytes, h.device, ws)
    _check(load_library().specvocab_dense_logits(_ptr(h), rows, d, ldh, _ptr(U), V, ldu, dt, _ptr(out),
                                                 _ptr(ws), 0 if ws is None else ws.numel(), _stream(stream)),
           "specvocab_dense_logits")
    return out
