"""CPU oracle for core attention over CA-task batches.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this package;
the HIP library and its Python binding never do, and this package imports nothing of theirs.

`ca_oracle.c` holds the arithmetic (the plain fp64 definition; see its header for the passages
it follows).  This file only compiles it with gcc and marshals numpy arrays into it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ca_oracle.c")
_LIB = os.path.join(_HERE, "libca_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile ca_oracle.c into libca_oracle.so next to it (gcc, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O3", "-mavx2", "-mfma", "-fopenmp", "-shared", "-fPIC", "-std=c11",
                               "-Wall", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _CBatch(ctypes.Structure):
    _fields_ = [
        ("n_docs", ctypes.c_int32), ("n_tasks", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
        ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("total_q", ctypes.c_int64), ("total_kv", ctypes.c_int64), ("scale", ctypes.c_double),
        ("doc_kv_start", ctypes.c_void_p), ("task_doc", ctypes.c_void_p),
        ("task_q_start", ctypes.c_void_p), ("task_q_len", ctypes.c_void_p),
        ("task_q_pos", ctypes.c_void_p), ("task_kv_len", ctypes.c_void_p),
    ]


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.ca_oracle_forward.restype = ctypes.c_int
        _lib.ca_oracle_backward.restype = ctypes.c_int
        _lib.ca_oracle_threads.restype = ctypes.c_int
        _lib.ca_oracle_merge.restype = ctypes.c_int
    return _lib


def threads() -> int:
    """Threads the oracle's OpenMP loops will use."""
    return int(_load().ca_oracle_threads())


def _batch_struct(batch, keep):
    def arr(x, dt):
        a = np.ascontiguousarray(np.asarray(x), dtype=dt)
        keep.append(a)
        return a.ctypes.data

    c = _CBatch()
    c.n_docs, c.n_tasks = batch.n_docs, batch.n_tasks
    c.n_q_heads, c.n_kv_heads, c.head_dim = batch.n_q_heads, batch.n_kv_heads, batch.head_dim
    c.total_q, c.total_kv, c.scale = batch.total_q, batch.total_kv, float(batch.scale)
    c.doc_kv_start = arr(batch.doc_kv_start, np.int64)
    c.task_doc = arr(batch.task_doc, np.int32)
    c.task_q_start = arr(batch.task_q_start, np.int64)
    c.task_q_len = arr(batch.task_q_len, np.int64)
    c.task_q_pos = arr(batch.task_q_pos, np.int64)
    c.task_kv_len = arr(batch.task_kv_len, np.int64)
    return c


def _f64(x, shape):
    a = np.ascontiguousarray(np.asarray(x, dtype=np.float64))
    if a.shape != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {a.shape}")
    return a


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data) if a is not None else ctypes.c_void_p(0)


def forward(batch, q, k, v):
    """O [total_q,Hq,D] and LSE [Hq,total_q] in fp64 for a batch descriptor (any object with the
    descriptor's field names and a `.scale`) and fp64-convertible Q, K, V arrays."""
    lib = _load()
    hq, hkv, d = batch.n_q_heads, batch.n_kv_heads, batch.head_dim
    q = _f64(q, (batch.total_q, hq, d))
    k = _f64(k, (batch.total_kv, hkv, d))
    v = _f64(v, (batch.total_kv, hkv, d))
    o = np.full((batch.total_q, hq, d), np.nan)
    lse = np.full((hq, batch.total_q), np.nan)
    keep = []
    c = _batch_struct(batch, keep)
    rc = lib.ca_oracle_forward(ctypes.byref(c), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse))
    if rc != 0:
        raise RuntimeError(f"ca_oracle_forward failed: {rc}")
    return o, lse


def backward(batch, q, k, v, o, d_o, lse, want=("dq", "dk", "dv")):
    """dQ, dK, dV (fp64; None for those not in `want`) and Delta [Hq,total_q]."""
    lib = _load()
    hq, hkv, d = batch.n_q_heads, batch.n_kv_heads, batch.head_dim
    q = _f64(q, (batch.total_q, hq, d))
    k = _f64(k, (batch.total_kv, hkv, d))
    v = _f64(v, (batch.total_kv, hkv, d))
    o = _f64(o, (batch.total_q, hq, d))
    d_o = _f64(d_o, (batch.total_q, hq, d))
    lse = _f64(lse, (hq, batch.total_q))
    dq = np.full_like(q, np.nan) if "dq" in want else None
    dk = np.full_like(k, np.nan) if "dk" in want else None
    dv = np.full_like(v, np.nan) if "dv" in want else None
    delta = np.full((hq, batch.total_q), np.nan)
    keep = []
    c = _batch_struct(batch, keep)
    rc = lib.ca_oracle_backward(ctypes.byref(c), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(d_o), _ptr(lse),
                                _ptr(dq), _ptr(dk), _ptr(dv), _ptr(delta))
    if rc != 0:
        raise RuntimeError(f"ca_oracle_backward failed: {rc}")
    return dq, dk, dv, delta


def forward_backward(batch, q, k, v, d_o, want=("dq", "dk", "dv")):
    o, lse = forward(batch, q, k, v)
    dq, dk, dv, delta = backward(batch, q, k, v, o, d_o, lse, want)
    return {"o": o, "lse": lse, "dq": dq, "dk": dk, "dv": dv, "delta": delta}


def merge_partials(part_rows, o_part, lse_part):
    """Combine partial results over disjoint key sets: part_rows [n_parts, n_rows] (row in the partial buffers,
    -1 = no such part), o_part [total_q_part, Hq, D], lse_part [Hq, total_q_part] -> O [n_rows, Hq, D], LSE [Hq, n_rows]."""
    lib = _load()
    pr = np.ascontiguousarray(np.asarray(part_rows), dtype=np.int64)
    n_parts, n_rows = pr.shape
    o_part = np.ascontiguousarray(np.asarray(o_part, dtype=np.float64))
    tq, hq, d = o_part.shape
    lse_part = _f64(lse_part, (hq, tq))
    if pr.size and (pr.max() >= tq or pr.min() < -1):
        raise ValueError("part_rows outside the partial buffers")
    o = np.full((n_rows, hq, d), np.nan)
    lse = np.full((hq, n_rows), np.nan)
    rc = lib.ca_oracle_merge(ctypes.c_int64(n_rows), ctypes.c_int32(n_parts), _ptr(pr), _ptr(o_part), _ptr(lse_part),
                             ctypes.c_int64(tq), ctypes.c_int32(hq), ctypes.c_int32(d), _ptr(o), _ptr(lse))
    if rc != 0:
        raise RuntimeError(f"ca_oracle_merge failed: {rc}")
    return o, lse
