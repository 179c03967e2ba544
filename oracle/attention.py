"""Python face of the C attention oracle (test infrastructure only).

Defines attention exactly as the plain formula in attention.c: per request,
per query head, softmax(scale * q k^T) v with a bottom-right aligned causal
mask and grouped-query head mapping kv_head = q_head // (Hq // Hkv)
(paper Sec. 2.1; Sec. 3 "lossless attention semantics").
"""
import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.build()
        _lib = ctypes.CDLL(path)
        _lib.oracle_attention_ragged.restype = ctypes.c_int
        _lib.oracle_attention_ragged.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double,
            ctypes.c_void_p, ctypes.c_int64,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
    return _lib


def _f32(x):
    if hasattr(x, "detach"):                      # torch tensor (any float dtype)
        x = x.detach().to("cpu").float().numpy()
    return np.ascontiguousarray(x, dtype=np.float32)


def attention_ragged(q, k, v, q_lens, kv_lens, scale, rows=None, return_lse=False,
                     nthreads=0):
    """q: [sum Lq, Hq, d]; k, v: [sum Lkv, Hkv, d] in request order.

    rows=None computes every output row -> [sum Lq, Hq, d] fp32.
    rows=[(request, head, t), ...] computes only those rows -> [len(rows), d].
    Returns (out[, lse], threads_used).
    """
    lib = _load()
    q, k, v = _f32(q), _f32(k), _f32(v)
    q_lens = np.asarray(q_lens, dtype=np.int64)
    kv_lens = np.asarray(kv_lens, dtype=np.int64)
    n = len(q_lens)
    qs = np.concatenate([[0], np.cumsum(q_lens)]).astype(np.int64)
    ks = np.concatenate([[0], np.cumsum(kv_lens)]).astype(np.int64)
    assert q.ndim == 3 and k.ndim == 3 and v.shape == k.shape
    assert q.shape[0] == qs[-1] and k.shape[0] == ks[-1]
    Hq, d = q.shape[1], q.shape[2]
    Hkv = k.shape[1]
    if rows is None:
        out = np.zeros_like(q)
        lse = np.zeros(q.shape[:2], dtype=np.float64) if return_lse else None
        rows_p, nrows = None, 0
    else:
        rows_a = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1, 3)
        out = np.zeros((rows_a.shape[0], d), dtype=np.float32)
        lse = np.zeros(rows_a.shape[0], dtype=np.float64) if return_lse else None
        rows_p, nrows = rows_a.ctypes.data, rows_a.shape[0]
    used = lib.oracle_attention_ragged(
        q.ctypes.data, k.ctypes.data, v.ctypes.data, qs.ctypes.data, ks.ctypes.data,
        n, Hq, Hkv, d, float(scale), rows_p, nrows,
        out.ctypes.data, None if lse is None else lse.ctypes.data, int(nthreads))
    if used < 0:
        raise ValueError("oracle_attention_ragged: bad arguments")
    if return_lse:
        return out, lse, used
    return out, used
