"""CPU oracle (test infrastructure, not product code).

Loads ``ns_oracle.c`` (built with gcc, OpenMP) through ctypes and exposes it
with numpy arguments.  Nothing here is imported by the HIP library or its
Python binding; only tests, the smoke check and the benchmark's CPU-baseline
leg use it.  All arithmetic lives in the C file (and, for the transformer
block, in ``vit_block.py``); this module only marshals arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ns_oracle.c")
_LIB = os.path.join(_HERE, "libns_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc if the library is missing or older than its source."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.oracle_count_pairs.restype = ctypes.c_int64
        _lib = lib
    return _lib


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _ptr(a, ct):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ct))


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def count_pairs(T, grid_w, block, radius=1, n_global=1, coords=None) -> int:
    c = None if coords is None else np.ascontiguousarray(coords, dtype=np.int32)
    return int(_load().oracle_count_pairs(
        ctypes.c_int(T), ctypes.c_int(n_global), ctypes.c_int(grid_w), ctypes.c_int(block),
        ctypes.c_int(radius), _ptr(c, ctypes.c_int32)))


def ns_attn(q, k, v, grid_h, grid_w, block, scale, radius=1, n_global=1, coords=None,
            rows=None, want_prob=False):
    """Neighbourhood-sparse attention by definition.

    q, k, v: [B,H,T,D] (any float dtype numpy can widen exactly to float32).
    Returns out float64 [B,H,T,D] (or [B,H,len(rows),D]) and, if want_prob, the
    softmax rows [B,H,n_out,T] with zeros at masked keys.
    """
    q, k, v = _f32(q), _f32(k), _f32(v)
    B, H, T, D = q.shape
    assert k.shape == q.shape and v.shape == q.shape
    c = None
    if coords is not None:
        c = np.ascontiguousarray(coords, dtype=np.int32)
        assert c.shape == (B, T - n_global)
    else:
        assert T == n_global + grid_h * grid_w
    r = None if rows is None else np.ascontiguousarray(rows, dtype=np.int32)
    nq = T if r is None else len(r)
    out = np.empty((B, H, nq, D), dtype=np.float64)
    prob = np.empty((B, H, nq, T), dtype=np.float64) if want_prob else None
    rc = _load().oracle_ns_attn(
        ctypes.c_int(B), ctypes.c_int(H), ctypes.c_int(T), ctypes.c_int(D),
        ctypes.c_int(n_global), ctypes.c_int(grid_h), ctypes.c_int(grid_w),
        ctypes.c_int(block), ctypes.c_int(radius), ctypes.c_double(scale),
        _ptr(q, ctypes.c_float), _ptr(k, ctypes.c_float), _ptr(v, ctypes.c_float),
        _ptr(c, ctypes.c_int32), _ptr(r, ctypes.c_int32), ctypes.c_int(0 if r is None else len(r)),
        _ptr(out, ctypes.c_double), _ptr(prob, ctypes.c_double))
    if rc != 0:
        raise ValueError("oracle_ns_attn: bad arguments")
    return (out, prob) if want_prob else out


def cls_scores(q, k, scale, n_global=1, want_logits=False):
    """Head-averaged softmax weight of the global query on every patch key: [B, T-G] float64."""
    q, k = _f32(q), _f32(k)
    B, H, T, D = q.shape
    scores = np.empty((B, T - n_global), dtype=np.float64)
    logits = np.empty((B, H, T), dtype=np.float64) if want_logits else None
    lse = np.empty((B, H), dtype=np.float64) if want_logits else None
    rc = _load().oracle_cls_scores(
        ctypes.c_int(B), ctypes.c_int(H), ctypes.c_int(T), ctypes.c_int(D),
        ctypes.c_int(n_global), ctypes.c_double(scale), _ptr(q, ctypes.c_float),
        _ptr(k, ctypes.c_float), _ptr(scores, ctypes.c_double), _ptr(logits, ctypes.c_double),
        _ptr(lse, ctypes.c_double))
    if rc != 0:
        raise ValueError("oracle_cls_scores: bad arguments")
    return (scores, logits, lse) if want_logits else scores


def topk(scores, k):
    """Indices of the k largest float32 scores per image, ties to the lower index, ascending."""
    s = _f32(scores)
    B, N = s.shape
    kept = np.empty((B, k), dtype=np.int32)
    rc = _load().oracle_topk(ctypes.c_int(B), ctypes.c_int(N), ctypes.c_int(k),
                             _ptr(s, ctypes.c_float), _ptr(kept, ctypes.c_int32))
    if rc != 0:
        raise ValueError("oracle_topk: bad arguments")
    return kept


def gather(x, kept, n_global=1):
    """Compaction: keep the global rows, then rows n_global + kept[b, t]; bit copy."""
    x = np.ascontiguousarray(x)
    kept = np.ascontiguousarray(kept, dtype=np.int32)
    B, T = x.shape[0], x.shape[1]
    k = kept.shape[1]
    N = T - n_global
    y = np.empty((B, n_global + k) + x.shape[2:], dtype=x.dtype)
    row_bytes = int(np.prod(x.shape[2:], dtype=np.int64)) * x.dtype.itemsize
    rc = _load().oracle_gather(ctypes.c_int(B), ctypes.c_int(N), ctypes.c_int(k),
                               ctypes.c_int(n_global), ctypes.c_size_t(row_bytes),
                               x.ctypes.data_as(ctypes.c_void_p), _ptr(kept, ctypes.c_int32),
                               y.ctypes.data_as(ctypes.c_void_p))
    if rc != 0:
        raise ValueError("oracle_gather: index out of range")
    return y
