"""TEST INFRASTRUCTURE ONLY -- the fp64 CPU checker for the hybrid-batch attention path.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py``
may import this package.  It imports nothing from the product package and shares no code
with it.

Contents
--------
``attention_oracle.c``    per-row softmax attention in double precision (paper section 2.1),
                          compiled here with gcc into ``liboracle.so``.
``kv_cache_reference.py`` what the paged K/V pools must hold after an append, and how a
                          sequence is read back through its block table (section 2.2, paged cache).
``scheduler_reference.py`` one iteration of stall-free batching (Algorithm 3, section 4.2).
``token_budget_reference.py`` the token budget chosen from a one-time profile (section 4.3).
``linear_oracle.c``       a linear layer over the batch's token rows in double precision
                          (sections 2.1 and 3.1), compiled into ``liblinear_oracle.so``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "attention_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib: Optional[ctypes.CDLL] = None
_LIN_SRC = os.path.join(_HERE, "linear_oracle.c")
_LIN_LIB = os.path.join(_HERE, "liblinear_oracle.so")
_lin_lib: Optional[ctypes.CDLL] = None


def build(force: bool = False) -> str:
    """Compile the C checker with gcc (-O2, OpenMP for row parallelism)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    stale = (not os.path.exists(_LIN_LIB)) or os.path.getmtime(_LIN_LIB) < os.path.getmtime(_LIN_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIN_LIB, _LIN_SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        i32p = ctypes.POINTER(ctypes.c_int32)
        i64p = ctypes.POINTER(ctypes.c_int64)
        f64p = ctypes.POINTER(ctypes.c_double)
        lib.oracle_hybrid_attention_window.restype = ctypes.c_int
        lib.oracle_hybrid_attention_window.argtypes = [
            u16p, u16p, u16p, i64p, i32p, i32p, i32p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double, ctypes.c_int,
            i32p, ctypes.c_int, f64p, ctypes.c_int]
        lib.oracle_softmax_weights.restype = ctypes.c_int
        lib.oracle_softmax_weights.argtypes = [
            u16p, u16p, i64p, i32p, i32p, i32p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double,
            ctypes.c_int, ctypes.c_int, f64p]
        lib.oracle_max_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _ptr(a: np.ndarray, ty):
    return a.ctypes.data_as(ctypes.POINTER(ty))


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def hybrid_attention(q_bits: np.ndarray, k_seq_bits: np.ndarray, v_seq_bits: np.ndarray,
                     kv_start: Sequence[int], q_start: Sequence[int], q_len: Sequence[int],
                     ctx_len: Sequence[int], sm_scale: float,
                     tokens: Optional[Sequence[int]] = None, num_threads: int = 0, window: int = 0) -> np.ndarray:
    """Attention of every (or the listed) batch row, all heads, in fp64.

    ``window`` > 0: sliding-window attention, the query at position p sees keys p-window+1 .. p.

    ``q_bits [T, Hq, d]``, ``k_seq_bits / v_seq_bits [sum(ctx_len), Hkv, d]`` are bf16 bit
    patterns (uint16); sequence ``s`` owns K/V rows ``kv_start[s] .. kv_start[s]+ctx_len[s]``.
    Returns ``[rows, Hq, d]`` float64.
    """
    lib = _load()
    q = np.ascontiguousarray(q_bits, dtype=np.uint16)
    k = np.ascontiguousarray(k_seq_bits, dtype=np.uint16)
    v = np.ascontiguousarray(v_seq_bits, dtype=np.uint16)
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    assert k.shape == v.shape and k.shape[2] == d
    kvs = np.ascontiguousarray(kv_start, dtype=np.int64)
    qs = np.ascontiguousarray(q_start, dtype=np.int32)
    ql = np.ascontiguousarray(q_len, dtype=np.int32)
    cl = np.ascontiguousarray(ctx_len, dtype=np.int32)
    S = ql.shape[0]
    assert int(kvs[-1]) + int(cl[-1]) <= k.shape[0] if S else True
    if tokens is None:
        tok = None
        n_rows = T
    else:
        tok = np.ascontiguousarray(tokens, dtype=np.int32)
        n_rows = tok.shape[0]
    out = np.empty((n_rows, Hq, d), dtype=np.float64)
    rc = lib.oracle_hybrid_attention_window(
        _ptr(q, ctypes.c_uint16), _ptr(k, ctypes.c_uint16), _ptr(v, ctypes.c_uint16),
        _ptr(kvs, ctypes.c_int64), _ptr(qs, ctypes.c_int32), _ptr(ql, ctypes.c_int32),
        _ptr(cl, ctypes.c_int32), S, T, Hq, Hkv, d, float(sm_scale), int(window),
        _ptr(tok, ctypes.c_int32) if tok is not None else None, n_rows,
        _ptr(out, ctypes.c_double), int(num_threads))
    if rc != 0:
        raise ValueError("oracle_hybrid_attention: inconsistent batch description")
    return out


def softmax_weights(q_bits, k_seq_bits, kv_start, q_start, q_len, ctx_len, sm_scale, token: int, head: int) -> np.ndarray:
    """Softmax weights of one (batch row, query head) over key positions 0..pos."""
    lib = _load()
    q = np.ascontiguousarray(q_bits, dtype=np.uint16)
    k = np.ascontiguousarray(k_seq_bits, dtype=np.uint16)
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    kvs = np.ascontiguousarray(kv_start, dtype=np.int64)
    qs = np.ascontiguousarray(q_start, dtype=np.int32)
    ql = np.ascontiguousarray(q_len, dtype=np.int32)
    cl = np.ascontiguousarray(ctx_len, dtype=np.int32)
    w = np.empty(int(cl.max()), dtype=np.float64)
    n = lib.oracle_softmax_weights(
        _ptr(q, ctypes.c_uint16), _ptr(k, ctypes.c_uint16), _ptr(kvs, ctypes.c_int64),
        _ptr(qs, ctypes.c_int32), _ptr(ql, ctypes.c_int32), _ptr(cl, ctypes.c_int32),
        ql.shape[0], Hq, Hkv, d, float(sm_scale), int(token), int(head), _ptr(w, ctypes.c_double))
    if n < 0:
        raise ValueError("token not in batch")
    return w[:n].copy()


def attention_for_batch(batch, tokens: Optional[Sequence[int]] = None, q_copy: int = 0,
                        num_threads: int = 0, kv=None, window: int = 0) -> np.ndarray:
    """Convenience: run the checker on a ``workloads.HybridBatch`` (duck-typed, not imported)."""
    k, v = kv if kv is not None else batch.kv_concat()
    return hybrid_attention(batch.q_bits(q_copy), k, v, batch.kv_start, batch.q_start, batch.q_len,
                            batch.ctx_len, batch.sm_scale, tokens=tokens, num_threads=num_threads, window=window)


def _load_linear() -> ctypes.CDLL:
    global _lin_lib
    if _lin_lib is None:
        build()
        lib = ctypes.CDLL(_LIN_LIB)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        i32p = ctypes.POINTER(ctypes.c_int32)
        lib.oracle_linear.restype = ctypes.c_int
        lib.oracle_linear.argtypes = [u16p, u16p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                      i32p, ctypes.c_int, i32p, ctypes.c_int,
                                      ctypes.POINTER(ctypes.c_double), ctypes.c_int]
        _lin_lib = lib
    return _lin_lib


def linear(x_bits: np.ndarray, w_bits: np.ndarray, rows: Optional[Sequence[int]] = None,
           cols: Optional[Sequence[int]] = None, num_threads: int = 0) -> np.ndarray:
    """``y[t, n] = sum_k x[t, k] * w[n, k]`` in fp64 for all (or the listed) token rows and output features.

    ``x_bits [T, K]`` and ``w_bits [N, K]`` are bf16 bit patterns (uint16).  Returns float64
    ``[len(rows) or T, len(cols) or N]``."""
    lib = _load_linear()
    x = np.ascontiguousarray(x_bits, dtype=np.uint16)
    w = np.ascontiguousarray(w_bits, dtype=np.uint16)
    if x.ndim != 2 or w.ndim != 2 or x.shape[1] != w.shape[1]:
        raise ValueError("x must be [T, K] and w [N, K]")
    T, K = x.shape
    N = w.shape[0]
    r = None if rows is None else np.ascontiguousarray(rows, dtype=np.int32)
    c = None if cols is None else np.ascontiguousarray(cols, dtype=np.int32)
    out = np.empty((T if r is None else len(r), N if c is None else len(c)), dtype=np.float64)
    rc = lib.oracle_linear(_ptr(x, ctypes.c_uint16), _ptr(w, ctypes.c_uint16), T, N, K,
                           None if r is None else _ptr(r, ctypes.c_int32), 0 if r is None else len(r),
                           None if c is None else _ptr(c, ctypes.c_int32), 0 if c is None else len(c),
                           _ptr(out, ctypes.c_double), num_threads)
    if rc != 0:
        raise ValueError("row or column index outside the matrices")
    return out
