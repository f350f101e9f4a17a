"""ctypes binding of the CPU oracle (oracle/si_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
the cpu_baseline leg of bench.py.  The product package never imports this.

All arrays are host numpy arrays.  q and K carry bfloat16 bit patterns as
uint16; w is float32.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from ctypes import POINTER, c_double, c_float, c_int32, c_int64, c_uint16, c_uint64

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "si_oracle.cpp")
_HDR = os.path.join(_HERE, "si_oracle.h")
_LIB = os.path.join(_HERE, "libsi_oracle.so")

MASK_NONE = 0
MASK_CAUSAL_BLOCK = 1


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (x86-64-v3 so the binary also runs on the GPU machine's host)."""
    stale = (
        force
        or not os.path.exists(_LIB)
        or os.path.getmtime(_LIB) < max(os.path.getmtime(_SRC), os.path.getmtime(_HDR))
    )
    if stale:
        cmd = [
            "g++", "-O2", "-std=c++17", "-march=x86-64-v3", "-fopenmp-simd", "-fPIC", "-shared",
            "-pthread", "-Wall", "-Wextra", "-o", _LIB, _SRC,
        ]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _p(arr, ctype):
    return arr.ctypes.data_as(POINTER(ctype))


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        L = ctypes.CDLL(_LIB)
        L.si_oracle_legal_count.restype = c_int64
        L.si_oracle_legal_count.argtypes = [c_int64, c_int64, c_int32, c_int32]
        L.si_oracle_score_row.restype = c_int32
        L.si_oracle_score_row.argtypes = [
            POINTER(c_uint16), POINTER(c_uint16), POINTER(c_float), c_int32, c_int32, c_int64,
            POINTER(c_double)]
        L.si_oracle_score_at.restype = c_int32
        L.si_oracle_score_at.argtypes = [
            POINTER(c_uint16), POINTER(c_uint16), POINTER(c_float), c_int32, c_int32,
            POINTER(c_int32), c_int64, POINTER(c_double)]
        L.si_oracle_sort_topk.restype = c_int32
        L.si_oracle_sort_topk.argtypes = [
            POINTER(c_double), c_int64, c_int32, POINTER(c_int32), POINTER(c_double)]
        L.si_oracle_topk_rows.restype = c_int32
        L.si_oracle_topk_rows.argtypes = [
            POINTER(c_uint16), POINTER(c_float), POINTER(c_uint16), POINTER(c_int32),
            POINTER(c_int64), c_int64, c_int32, c_int32, c_int64, c_int32, c_int32, c_int32,
            POINTER(c_int32), POINTER(c_double), c_int32]
        L.si_oracle_sparse_attention_rows.restype = c_int32
        L.si_oracle_sparse_attention_rows.argtypes = [
            POINTER(c_uint16), POINTER(c_uint16), POINTER(c_int32), POINTER(c_int32), POINTER(c_int64),
            c_int64, c_int32, c_int32, c_int64, c_int32, c_int32, c_int32, c_int32, c_double,
            POINTER(c_double), c_int32]
        L.si_oracle_stream_topk.restype = c_int32
        L.si_oracle_stream_topk.argtypes = [
            POINTER(c_double), c_int64, POINTER(c_int64), c_int32, POINTER(c_int32),
            POINTER(c_double)]
        L.si_oracle_chunked_topk_row.restype = c_int32
        L.si_oracle_chunked_topk_row.argtypes = [
            POINTER(c_double), c_int64, c_int64, c_int32, c_int64, c_int32, POINTER(c_int32),
            POINTER(c_double)]
        L.si_oracle_materialize_bytes.restype = c_uint64
        L.si_oracle_materialize_bytes.argtypes = [c_int64] * 4
        L.si_oracle_mask_bytes.restype = c_uint64
        L.si_oracle_mask_bytes.argtypes = [c_int64] * 3
        _lib = L
    return _lib


def _u16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def legal_count(t: int, T: int, m: int, mask_mode: int) -> int:
    return int(lib().si_oracle_legal_count(t, T, m, mask_mode))


def score_row(q_row, K, w_row, n_keys=None):
    """fp64 scores of one query ([H,D] uint16) against K[:n_keys] ([T,D] uint16)."""
    q_row, K, w_row = _u16(q_row), _u16(K), _f32(w_row)
    H, D = q_row.shape
    assert K.ndim == 2 and K.shape[1] == D and w_row.shape == (H,)
    n = K.shape[0] if n_keys is None else int(n_keys)
    assert 0 <= n <= K.shape[0]
    out = np.empty(n, dtype=np.float64)
    rc = lib().si_oracle_score_row(_p(q_row, c_uint16), _p(K, c_uint16), _p(w_row, c_float),
                                   H, D, n, _p(out, c_double))
    assert rc == 0, rc
    return out


def score_at(q_row, K, w_row, idx):
    q_row, K, w_row = _u16(q_row), _u16(K), _f32(w_row)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    H, D = q_row.shape
    assert K.ndim == 2 and K.shape[1] == D and w_row.shape == (H,)
    assert idx.size == 0 or idx.max() < K.shape[0]
    out = np.empty(idx.shape, dtype=np.float64)
    rc = lib().si_oracle_score_at(_p(q_row, c_uint16), _p(K, c_uint16), _p(w_row, c_float),
                                  H, D, _p(idx, c_int32), idx.size, _p(out, c_double))
    assert rc == 0, rc
    return out


def sort_topk(scores, k: int):
    scores = np.ascontiguousarray(scores, dtype=np.float64)
    idx = np.empty(k, dtype=np.int32)
    sc = np.empty(k, dtype=np.float64)
    rc = lib().si_oracle_sort_topk(_p(scores, c_double), scores.size, k, _p(idx, c_int32),
                                   _p(sc, c_double))
    assert rc == 0, rc
    return idx, sc


def topk_rows(q_rows, w_rows, K, b_of_row, t_of_row, m: int, k: int, mask_mode: int,
              n_threads: int = 1):
    """Top-k of the listed query rows.  q_rows [n,H,D] uint16, w_rows [n,H], K [B,T,D] uint16."""
    q_rows, K, w_rows = _u16(q_rows), _u16(K), _f32(w_rows)
    b_of_row = np.ascontiguousarray(b_of_row, dtype=np.int32)
    t_of_row = np.ascontiguousarray(t_of_row, dtype=np.int64)
    n, H, D = q_rows.shape
    B, T, D2 = K.shape
    assert D2 == D and w_rows.shape == (n, H) and b_of_row.shape == (n,) and t_of_row.shape == (n,)
    assert n == 0 or (0 <= b_of_row.min() and b_of_row.max() < B and t_of_row.min() >= 0)
    idx = np.empty((n, k), dtype=np.int32)
    sc = np.empty((n, k), dtype=np.float64)
    rc = lib().si_oracle_topk_rows(
        _p(q_rows, c_uint16), _p(w_rows, c_float), _p(K, c_uint16), _p(b_of_row, c_int32),
        _p(t_of_row, c_int64), n, H, D, T, m, k, mask_mode, _p(idx, c_int32), _p(sc, c_double),
        n_threads)
    assert rc == 0, rc
    return idx, sc


def topk_all(q, K, w, m: int, k: int, mask_mode: int, n_threads: int = 1):
    """Every row of a whole problem.  q [B,S,H,D] uint16, K [B,T,D] uint16, w [B,S,H]."""
    q = _u16(q)
    B, S, H, D = q.shape
    b = np.repeat(np.arange(B, dtype=np.int32), S)
    t = np.tile(np.arange(S, dtype=np.int64), B)
    idx, sc = topk_rows(q.reshape(B * S, H, D), _f32(w).reshape(B * S, H), K, b, t, m, k,
                        mask_mode, n_threads)
    return idx.reshape(B, S, k), sc.reshape(B, S, k)


def sparse_attention_rows(qa_rows, K, idx_rows, b_of_row, t_of_row, m: int, mask_mode: int,
                          n_win: int, scale: float, n_threads: int = 1):
    """Attention of the listed query rows over TopK(t) U Window(t) (see si_oracle.h).
    qa_rows [n,H,D] uint16, K [B,T,D] uint16, idx_rows [n,k] int32 -> [n,H,D] float64."""
    qa_rows, K = _u16(qa_rows), _u16(K)
    idx_rows = np.ascontiguousarray(idx_rows, dtype=np.int32)
    b_of_row = np.ascontiguousarray(b_of_row, dtype=np.int32)
    t_of_row = np.ascontiguousarray(t_of_row, dtype=np.int64)
    n, H, D = qa_rows.shape
    B, T, D2 = K.shape
    k = idx_rows.shape[1]
    assert D2 == D and idx_rows.shape == (n, k) and b_of_row.shape == (n,) and t_of_row.shape == (n,)
    assert n == 0 or (0 <= b_of_row.min() and b_of_row.max() < B and t_of_row.min() >= 0)
    out = np.empty((n, H, D), dtype=np.float64)
    rc = lib().si_oracle_sparse_attention_rows(
        _p(qa_rows, c_uint16), _p(K, c_uint16), _p(idx_rows, c_int32), _p(b_of_row, c_int32),
        _p(t_of_row, c_int64), n, H, D, T, m, k, mask_mode, n_win, float(scale), _p(out, c_double),
        n_threads)
    if rc == -2:
        raise ValueError("index outside [-1, T)")
    assert rc == 0, rc
    return out


def stream_topk(scores, perm, k: int):
    scores = np.ascontiguousarray(scores, dtype=np.float64)
    perm = np.ascontiguousarray(perm, dtype=np.int64)
    assert perm.shape == scores.shape
    idx = np.empty(k, dtype=np.int32)
    sc = np.empty(k, dtype=np.float64)
    rc = lib().si_oracle_stream_topk(_p(scores, c_double), scores.size, _p(perm, c_int64), k,
                                     _p(idx, c_int32), _p(sc, c_double))
    assert rc == 0, rc
    return idx, sc


def chunked_topk_row(scores, legal: int, k: int, c_T: int, variant: int = 0):
    scores = np.ascontiguousarray(scores, dtype=np.float64)
    idx = np.empty(k, dtype=np.int32)
    sc = np.empty(k, dtype=np.float64)
    rc = lib().si_oracle_chunked_topk_row(_p(scores, c_double), scores.size, legal, k, c_T,
                                          variant, _p(idx, c_int32), _p(sc, c_double))
    assert rc == 0, rc
    return idx, sc


def materialize_bytes(B: int, S: int, H: int, T: int) -> int:
    return int(lib().si_oracle_materialize_bytes(B, S, H, T))


def mask_bytes(B: int, S: int, T: int) -> int:
    return int(lib().si_oracle_mask_bytes(B, S, T))
