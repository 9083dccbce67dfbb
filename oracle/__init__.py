"""ctypes front end of the CPU oracle (oracle/specvocab_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
benchmark's cpu_baseline leg.  The HIP library and its Python binding never
import this package, and this package never imports them.

Arrays: float32 inputs are numpy float32; bfloat16 inputs are numpy uint16 bit
patterns.  All floating-point results are numpy float64 (see the C file for why).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "specvocab_oracle.c")
_LIB = os.path.join(_HERE, "libspecvocab_oracle.so")

F32, BF16 = 0, 1
PER_ROW, PER_STEP = 0, 1
ACC_F32, ACC_F64 = 0, 1

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no FMA contraction so that the float32 mode rounds
    after every multiply and every add, as written)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-std=c11", "-shared", "-fPIC",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.svo_mac_count.restype = ctypes.c_uint64
        lib.svo_reset_mac_count.restype = None
        for name in ("svo_dense_logits", "svo_subset_logits", "svo_select", "svo_softmax_topk", "svo_log_softmax"):
            getattr(lib, name).restype = ctypes.c_int
        _lib = lib
    return _lib


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError(f"oracle inputs must be float32 or uint16 (bf16 bits), got {a.dtype}")


def _acc_code(acc: str) -> int:
    return {"f32": ACC_F32, "f64": ACC_F64}[acc]


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(rc: int, what: str):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def _same_dtype(*arrs):
    code = _dtype_code(arrs[0])
    for a in arrs[1:]:
        if _dtype_code(a) != code:
            raise TypeError("all matrices of one call must share a storage dtype")
    return code


def _c2(a: np.ndarray) -> np.ndarray:
    """A matrix whose rows are contiguous; a row stride larger than the row length (a view
    into a wider matrix) is kept and handed to the C side as the leading dimension."""
    a = np.asarray(a)
    if a.ndim == 1:
        a = a.reshape(1, -1)
    if a.ndim != 2:
        raise ValueError("expected a matrix")
    item = a.dtype.itemsize
    ok = a.strides[1] == item and a.strides[0] % item == 0 and a.strides[0] >= a.shape[1] * item
    if a.shape[0] == 1 and a.strides[1] == item:
        ok = True
    if not ok:
        a = np.ascontiguousarray(a)
    return a


def _ld(a: np.ndarray) -> int:
    if a.shape[0] == 1:
        return a.shape[1]
    return a.strides[0] // a.dtype.itemsize


def reset_mac_count() -> None:
    _load().svo_reset_mac_count()


def mac_count() -> int:
    return int(_load().svo_mac_count())


def dense_logits(h: np.ndarray, U: np.ndarray, acc: str = "f32") -> np.ndarray:
    """z = U h for every row of h (Section 3.1). Returns [rows x V] float64."""
    h, U = _c2(h), _c2(U)
    dt = _same_dtype(h, U)
    rows, d = h.shape
    V, d2 = U.shape
    if d2 != d:
        raise ValueError("U and h disagree on d")
    out = np.empty((rows, V), dtype=np.float64)
    rc = _load().svo_dense_logits(_ptr(h), ctypes.c_int64(rows), ctypes.c_int64(d), ctypes.c_int64(_ld(h)),
                                  _ptr(U), ctypes.c_int64(V), ctypes.c_int64(_ld(U)), dt, _acc_code(acc),
                                  _ptr(out))
    _check(rc, "dense_logits")
    return out


def subset_logits(h: np.ndarray, U: np.ndarray, idx: np.ndarray, acc: str = "f32") -> np.ndarray:
    """z'[r, j] = <U[idx(r, j)], h_r> (Section 3.3 Step 3). idx [rows x k] or [k] (one set per
    step). Returns [rows x k] float64."""
    h, U = _c2(h), _c2(U)
    dt = _same_dtype(h, U)
    rows, d = h.shape
    V, d2 = U.shape
    if d2 != d:
        raise ValueError("U and h disagree on d")
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    if idx.ndim == 1:
        mode, k = PER_STEP, idx.shape[0]
    else:
        if idx.shape[0] != rows:
            raise ValueError("per-row idx needs one row per hidden state")
        mode, k = PER_ROW, idx.shape[1]
    out = np.empty((rows, k), dtype=np.float64)
    rc = _load().svo_subset_logits(_ptr(h), ctypes.c_int64(rows), ctypes.c_int64(d), ctypes.c_int64(_ld(h)),
                                   _ptr(U), ctypes.c_int64(V), ctypes.c_int64(_ld(U)), dt,
                                   _ptr(idx), ctypes.c_int64(k), mode, _acc_code(acc), _ptr(out))
    _check(rc, "subset_logits")
    return out


def select(h: np.ndarray, W_down: np.ndarray, W_vocab: np.ndarray, k: int,
           hprime_round: Optional[bool] = None, acc: str = "f32", full: bool = False,
           tau: Optional[float] = None):
    """Steps 1-2 of Section 3.3. Returns (idx [rows x k] int32 ascending, scores [rows x k]) and,
    with full=True, also (s [rows x V], h' [rows x d']).  hprime_round defaults to True for bf16
    storage and False for float32.  With tau, selected tokens scoring below tau become padding
    slots (id -1, score -inf) in place."""
    h = _c2(h)
    W_down, W_vocab = np.ascontiguousarray(_c2(W_down)), np.ascontiguousarray(_c2(W_vocab))
    dt = _same_dtype(h, W_down, W_vocab)
    rows, d = h.shape
    d_prime, d2 = W_down.shape
    V, dp2 = W_vocab.shape
    if d2 != d or dp2 != d_prime:
        raise ValueError("selector shapes disagree")
    if hprime_round is None:
        hprime_round = dt == BF16
    idx = np.empty((rows, k), dtype=np.int32)
    scores = np.empty((rows, k), dtype=np.float64)
    s_full = np.empty((rows, V), dtype=np.float64) if full else None
    hp = np.empty((rows, d_prime), dtype=np.float64) if full else None
    rc = _load().svo_select(_ptr(h), ctypes.c_int64(rows), ctypes.c_int64(d), ctypes.c_int64(_ld(h)),
                            _ptr(W_down), ctypes.c_int64(d_prime), _ptr(W_vocab), ctypes.c_int64(V),
                            dt, int(bool(hprime_round)), _acc_code(acc), ctypes.c_int64(k),
                            ctypes.c_double(-np.inf if tau is None else float(tau)),
                            _ptr(idx), _ptr(scores), _ptr(s_full), _ptr(hp))
    _check(rc, "select")
    if full:
        return idx, scores, s_full, hp
    return idx, scores


def softmax_topk(logits: np.ndarray, idx: np.ndarray, kd: int, full: bool = False):
    """Subset softmax + top-kd draft tokens. logits [rows x k] (cast to float32, the hand-over
    precision); idx [rows x k] or [k]. Returns (tok [rows x kd] int32, prob [rows x kd] float64)
    and, with full=True, also q_K [rows x k]."""
    z = np.ascontiguousarray(_c2(np.asarray(logits)), dtype=np.float32)
    rows, k = z.shape
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    if idx.ndim == 1:
        mode = PER_STEP
        if idx.shape[0] != k:
            raise ValueError("idx and logits disagree on k")
    else:
        mode = PER_ROW
        if idx.shape != (rows, k):
            raise ValueError("idx and logits disagree on shape")
    tok = np.empty((rows, kd), dtype=np.int32)
    prob = np.empty((rows, kd), dtype=np.float64)
    q = np.empty((rows, k), dtype=np.float64) if full else None
    rc = _load().svo_softmax_topk(_ptr(z), _ptr(idx), mode, ctypes.c_int64(rows), ctypes.c_int64(k),
                                  ctypes.c_int64(kd), _ptr(tok), _ptr(prob), _ptr(q))
    _check(rc, "softmax_topk")
    if full:
        return tok, prob, q
    return tok, prob


def log_softmax(s: np.ndarray) -> np.ndarray:
    """Section 3.4: log q_aux = log softmax(s) over the whole vocabulary, row by row, in float64."""
    s = np.ascontiguousarray(np.atleast_2d(np.asarray(s, dtype=np.float64)))
    rows, V = s.shape
    out = np.empty((rows, V), dtype=np.float64)
    rc = _load().svo_log_softmax(_ptr(s), ctypes.c_int64(rows), ctypes.c_int64(V), _ptr(out))
    _check(rc, "log_softmax")
    return out


def aux_log_softmax(h: np.ndarray, W_down: np.ndarray, W_vocab: np.ndarray,
                    hprime_round: Optional[bool] = None, acc: str = "f32") -> np.ndarray:
    """Section 3.4: log q_aux(x_t | x_<t) = log softmax(W_vocab (W_down h_t)), [rows x V] float64.
    The scores are those of Section 3.3 Step 1 (same rounding of h' as select)."""
    _, _, s_full, _ = select(h, W_down, W_vocab, 1, hprime_round=hprime_round, acc=acc, full=True)
    return log_softmax(s_full)

