"""Attention oracle: every head attends to its own selected frames plus the chunk.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).

The arithmetic lives in ``attention.c`` (Eq. 1 written out, double
accumulation).  This file only assembles, per head, the key/value sequence
``[selected history frames in ascending id order || current chunk]`` (Eq. 2 and
Sec. 4.3: each batch-head pair has its own effective length) and hands it to C.
"""
import ctypes
import math

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(_build.build())
        lib.pfo_attn_head.restype = ctypes.c_int
        lib.pfo_attn_head.argtypes = [ctypes.c_void_p] * 4 + [ctypes.c_int] * 3 + \
            [ctypes.c_double, ctypes.c_void_p, ctypes.c_void_p]
        lib.pfo_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads():
    return int(_load().pfo_num_threads())


def widen_bf16(bits):
    """uint16 bf16 bit patterns -> the float32 with the same value."""
    return (np.asarray(bits, np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def attn_head(q, K, V, rows=None, scale=None, return_weights=False):
    """q [Lq, D], K/V [Lkv, D] float32 -> out [n_rows, D] float32 (and weights [n_rows, Lkv] float64).

    ``rows`` restricts the evaluation to some query rows (sampled parity at full size)."""
    q = np.ascontiguousarray(q, np.float32)
    K = np.ascontiguousarray(K, np.float32)
    V = np.ascontiguousarray(V, np.float32)
    Lq, D = q.shape
    Lkv = K.shape[0]
    assert K.shape == (Lkv, D) and V.shape == (Lkv, D)
    if scale is None:
        scale = 1.0 / math.sqrt(D)
    if rows is None:
        rows_arr, n_rows, rows_ptr = None, Lq, None
    else:
        rows_arr = np.ascontiguousarray(rows, np.int32)
        assert rows_arr.ndim == 1 and (rows_arr >= 0).all() and (rows_arr < Lq).all()
        n_rows, rows_ptr = rows_arr.size, rows_arr.ctypes.data
    out = np.empty((n_rows, D), np.float32)
    w = np.empty((n_rows, Lkv), np.float64) if return_weights else None
    rc = _load().pfo_attn_head(q.ctypes.data, K.ctypes.data, V.ctypes.data, rows_ptr, n_rows, Lkv, D,
                               float(scale), out.ctypes.data, None if w is None else w.ctypes.data)
    if rc != 0:
        raise RuntimeError("pfo_attn_head failed")
    return (out, w) if return_weights else out


def ragged_attention(q, history, k_cur, v_cur, rows=None, scale=None):
    """All heads.  q, k_cur, v_cur: float32 [H, Lq, D].  ``history[h]`` = (K_hist, V_hist), float32
    [n_sel[h]*tpf, D]: head h's selected history frames, already concatenated in ascending frame id.
    Returns float32 [H, n_rows, D]."""
    H = q.shape[0]
    outs = []
    for h in range(H):
        Kh = np.concatenate([history[h][0], k_cur[h]], 0)
        Vh = np.concatenate([history[h][1], v_cur[h]], 0)
        outs.append(attn_head(q[h], Kh, Vh, rows=rows, scale=scale))
    return np.stack(outs, 0)
