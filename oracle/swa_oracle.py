"""ctypes front end of the fp64 CPU oracle (``swa_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by the tests, by ``__graft_entry__.smoke()``
and by the ``cpu_baseline`` leg of ``bench.py``.  The HIP library and its Python
binding never import this module, and this module imports nothing of theirs.

All floating-point arrays are C-contiguous ``float64`` numpy arrays, all index
arrays ``int32``.  Shapes follow the header of ``swa_oracle.c``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "swa_oracle.c")
_LIB = os.path.join(_HERE, "libswa_oracle.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile ``swa_oracle.c`` with gcc (-O2, OpenMP) into ``libswa_oracle.so``."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _pd(a):
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _pi(a):
    assert a.dtype == np.int32 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.swa_oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(lib().swa_oracle_num_threads())


def set_num_threads(t: int) -> None:
    lib().swa_oracle_set_num_threads(ctypes.c_int(t))


def budget(n: int, m: int, w: int, sparsity_bp: int):
    """(keep, n_local, n_global) for logical length n, cached length m."""
    keep, nl, ng = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    lib().swa_oracle_budget(ctypes.c_int32(n), ctypes.c_int32(m), ctypes.c_int32(w),
                            ctypes.c_int32(sparsity_bp), ctypes.byref(keep), ctypes.byref(nl),
                            ctypes.byref(ng))
    return keep.value, nl.value, ng.value


def _dims(K):
    b, h, cap, d = K.shape
    return ctypes.c_int32(b), ctypes.c_int32(h), ctypes.c_int32(d), ctypes.c_int32(cap)


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def append(k_new, v_new, K, V, score, pos, cache_len, seq_len) -> None:
    """In place: K, V, score, pos, cache_len."""
    b, h, d, cap = _dims(K)
    rc = lib().swa_oracle_append(b, h, d, cap, _pd(_f64(k_new)), _pd(_f64(v_new)), _pd(K), _pd(V),
                                 _pd(score), _pi(pos), _pi(cache_len), _pi(_i32(seq_len)))
    _check(rc, "append")


def probs(q, K, cache_len, scale: float):
    b, h, d, cap = _dims(K)
    p = np.zeros(K.shape[:3], dtype=np.float64)
    lib().swa_oracle_probs(b, h, d, cap, ctypes.c_double(scale), _pd(_f64(q)), _pd(K),
                           _pi(_i32(cache_len)), _pd(p))
    return p


def accumulate(p, cache_len, score) -> None:
    """In place: score."""
    b, h, cap = p.shape
    lib().swa_oracle_accumulate(ctypes.c_int32(b), ctypes.c_int32(h), ctypes.c_int32(cap), _pd(p),
                                _pi(_i32(cache_len)), _pd(score))


def select(score, cache_len, seq_len, w: int, sparsity_bp: int, head_shared: bool = False):
    """Returns (kept_idx [b,h,cap] padded with -1, kept_cnt [b])."""
    score = _f64(score)
    b, h, cap = score.shape
    kept_idx = np.full((b, h, cap), -1, dtype=np.int32)
    kept_cnt = np.zeros((b,), dtype=np.int32)
    fn = lib().swa_oracle_select_shared if head_shared else lib().swa_oracle_select
    rc = fn(ctypes.c_int32(b), ctypes.c_int32(h), ctypes.c_int32(cap),
                                 ctypes.c_int32(w), ctypes.c_int32(sparsity_bp), _pd(score),
                                 _pi(_i32(cache_len)), _pi(_i32(seq_len)), _pi(kept_idx),
                                 _pi(kept_cnt))
    _check(rc, "select")
    return kept_idx, kept_cnt


def sparse_attention(q, K, V, kept_idx, kept_cnt, scale: float):
    b, h, d, cap = _dims(K)
    out = np.zeros((K.shape[0], K.shape[1], K.shape[3]), dtype=np.float64)
    rc = lib().swa_oracle_sparse_attention(b, h, d, cap, ctypes.c_double(scale), _pd(_f64(q)),
                                           _pd(K), _pd(V), _pi(_i32(kept_idx)),
                                           _pi(_i32(kept_cnt)), _pd(out))
    _check(rc, "sparse_attention")
    return out


def compact(K, V, score, pos, kept_idx, kept_cnt, cache_len) -> None:
    """In place: K, V, score, pos, cache_len."""
    b, h, d, cap = _dims(K)
    rc = lib().swa_oracle_compact(b, h, d, cap, _pd(K), _pd(V), _pd(score), _pi(pos),
                                  _pi(_i32(kept_idx)), _pi(_i32(kept_cnt)), _pi(cache_len))
    _check(rc, "compact")


def decode_step(q, k_new, v_new, K, V, score, pos, cache_len, seq_len, w: int, sparsity_bp: int,
                scale: float, want_probs: bool = True, head_shared: bool = False):
    """One full step.  In place: K, V, score, pos, cache_len.

    Returns (kept_idx, kept_cnt, out, probs or None).
    """
    b, h, d, cap = _dims(K)
    kept_idx = np.full(K.shape[:3], -1, dtype=np.int32)
    kept_cnt = np.zeros((K.shape[0],), dtype=np.int32)
    out = np.zeros((K.shape[0], K.shape[1], K.shape[3]), dtype=np.float64)
    p = np.zeros(K.shape[:3], dtype=np.float64) if want_probs else None
    rc = lib().swa_oracle_decode_step(
        b, h, d, cap, ctypes.c_int32(w), ctypes.c_int32(sparsity_bp), ctypes.c_double(scale),
        _pd(_f64(q)), _pd(_f64(k_new)), _pd(_f64(v_new)), _pd(K), _pd(V), _pd(score), _pi(pos),
        _pi(cache_len), _pi(_i32(seq_len)), _pi(kept_idx), _pi(kept_cnt), _pd(out),
        _pd(p) if want_probs else None, ctypes.c_int32(1 if head_shared else 0))
    _check(rc, "decode_step")
    return kept_idx, kept_cnt, out, p


def prefill_scores(q_tail, K, cache_len, scale: float):
    """q_tail [b,h,R,d] -> score [b,h,cap]."""
    b, h, d, cap = _dims(K)
    q_tail = _f64(q_tail)
    R = q_tail.shape[2]
    score = np.zeros(K.shape[:3], dtype=np.float64)
    rc = lib().swa_oracle_prefill_scores(b, h, d, cap, ctypes.c_int32(R), ctypes.c_double(scale),
                                         _pd(q_tail), _pd(K), _pi(_i32(cache_len)), _pd(score))
    _check(rc, "prefill_scores")
    return score


def _pf(a):
    assert a.dtype == np.float32 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _pu8(a):
    assert a.dtype == np.uint8 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))


def _rows_dims(X):
    b, h, rows, d = X.shape
    return ctypes.c_int32(b), ctypes.c_int32(h), ctypes.c_int32(d), ctypes.c_int32(rows)


def kv_qparams(X, count):
    """Channel-wise scale and zero point, fp32 [b,h,d] each, over rows 0..count[s]-1 of X [b,h,rows,d]."""
    X = _f64(X)
    b, h, d, rows = _rows_dims(X)
    lam = np.zeros((X.shape[0], X.shape[1], X.shape[3]), dtype=np.float32)
    zero = np.zeros_like(lam)
    lib().swa_oracle_kv_qparams(b, h, d, rows, _pd(X), _pi(_i32(count)), _pf(lam), _pf(zero))
    return lam, zero


def kv_quantize(X, count, lam, zero):
    """uint8 codes [b,h,rows,d] of the valid rows of X (the rest 0)."""
    X = _f64(X)
    b, h, d, rows = _rows_dims(X)
    codes = np.zeros(X.shape, dtype=np.uint8)
    lib().swa_oracle_kv_quantize(b, h, d, rows, _pd(X), _pi(_i32(count)),
                                 _pf(np.ascontiguousarray(lam, dtype=np.float32)),
                                 _pf(np.ascontiguousarray(zero, dtype=np.float32)), _pu8(codes))
    return codes


def kv_dequantize(codes, count, lam, zero):
    """float64 [b,h,rows,d]: scale * (code - zero) on the valid rows (the rest 0)."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    b, h, d, rows = _rows_dims(codes)
    X = np.zeros(codes.shape, dtype=np.float64)
    lib().swa_oracle_kv_dequantize(b, h, d, rows, _pu8(codes), _pi(_i32(count)),
                                   _pf(np.ascontiguousarray(lam, dtype=np.float32)),
                                   _pf(np.ascontiguousarray(zero, dtype=np.float32)), _pd(X))
    return X


def prefill_rows(q_tail, K, cache_len, scale: float):
    """q_tail [b,h,R,d] -> ring [b,h,R,cap]: the last R rows of the prompt's causal attention weights."""
    b, h, d, cap = _dims(K)
    q_tail = _f64(q_tail)
    R = q_tail.shape[2]
    ring = np.zeros((K.shape[0], K.shape[1], R, K.shape[2]), dtype=np.float64)
    rc = lib().swa_oracle_prefill_rows(b, h, d, cap, ctypes.c_int32(R), ctypes.c_double(scale),
                                       _pd(q_tail), _pd(K), _pi(_i32(cache_len)), _pd(ring))
    _check(rc, "prefill_rows")
    return ring


def compact_ring(ring, kept_idx, kept_cnt) -> None:
    """In place: the ring's columns follow the kept tokens."""
    b, h, R, cap = ring.shape
    rc = lib().swa_oracle_compact_ring(ctypes.c_int32(b), ctypes.c_int32(h), ctypes.c_int32(cap),
                                       ctypes.c_int32(R), _pd(ring), _pi(_i32(kept_idx)),
                                       _pi(_i32(kept_cnt)))
    _check(rc, "compact_ring")


def decode_step_window(q, k_new, v_new, K, V, ring, row: int, score, pos, cache_len, seq_len, w: int,
                       sparsity_bp: int, scale: float, head_shared: bool = False):
    """One step with the strict local attention sum.  In place: K, V, ring, score, pos, cache_len.

    Returns (kept_idx, kept_cnt, out, probs).
    """
    b, h, d, cap = _dims(K)
    R = ring.shape[2]
    kept_idx = np.full(K.shape[:3], -1, dtype=np.int32)
    kept_cnt = np.zeros((K.shape[0],), dtype=np.int32)
    out = np.zeros((K.shape[0], K.shape[1], K.shape[3]), dtype=np.float64)
    p = np.zeros(K.shape[:3], dtype=np.float64)
    rc = lib().swa_oracle_decode_step_window(
        b, h, d, cap, ctypes.c_int32(w), ctypes.c_int32(sparsity_bp), ctypes.c_double(scale),
        ctypes.c_int32(R), ctypes.c_int32(row), _pd(_f64(q)), _pd(_f64(k_new)), _pd(_f64(v_new)),
        _pd(K), _pd(V), _pd(ring), _pd(score), _pi(pos), _pi(cache_len), _pi(_i32(seq_len)),
        _pi(kept_idx), _pi(kept_cnt), _pd(out), _pd(p), ctypes.c_int32(1 if head_shared else 0))
    _check(rc, "decode_step_window")
    return kept_idx, kept_cnt, out, p


def prefill_attention(Q, K, V, cache_len, scale: float):
    """Causal attention over the prompt: Q, K, V [b,h,cap,d] -> out [b,h,cap,d] (rows >= cache_len zero)."""
    b, h, d, cap = _dims(K)
    out = np.zeros(K.shape, dtype=np.float64)
    rc = lib().swa_oracle_prefill_attention(b, h, d, cap, ctypes.c_double(scale), _pd(_f64(Q)), _pd(K),
                                            _pd(V), _pi(_i32(cache_len)), _pd(out))
    _check(rc, "prefill_attention")
    return out
