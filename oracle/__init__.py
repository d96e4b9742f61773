"""CPU fp64 oracle (test infrastructure only).

Python face of ``prism_oracle.c``: the page-table writer and textbook causal
softmax attention over prefix + suffix read through the block table (paper
Sec. 2.2, Eq. 3-4).  Only tests, the smoke check and the benchmark's
CPU-baseline leg may import this package; the GPU library never does, and this
package imports nothing from the GPU library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "prism_oracle.c")
_LIB = os.path.join(_HERE, "libprism_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no fast-math, OpenMP over rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.prism_oracle_threads.restype = ctypes.c_int
    return _lib


def threads() -> int:
    return int(_load().prism_oracle_threads())


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _u16(a: np.ndarray) -> np.ndarray:
    assert a.dtype == np.uint16
    return np.ascontiguousarray(a)


def kv_append(k_src, v_src, k_pool, v_pool, block_table, prefix_len, suffix_len):
    """Return copies of (k_pool, v_pool) with the suffix rows written in.

    k_src, v_src: uint16 [sum_S, Hkv, d]; pools: uint16 [pages, Hkv, page, d]."""
    k_src, v_src = _u16(k_src), _u16(v_src)
    k_out, v_out = _u16(k_pool).copy(), _u16(v_pool).copy()
    bt, pl, sl = _i32(block_table), _i32(prefix_len), _i32(suffix_len)
    _, Hkv, page, d = k_out.shape
    assert k_src.shape[0] == int(sl.sum()) and k_src.shape[1:] == (Hkv, d)
    _load().prism_oracle_kv_append(_p(k_src), _p(v_src), _p(k_out), _p(v_out), _p(bt), _p(pl), _p(sl),
                                   ctypes.c_int(bt.shape[0]), ctypes.c_int(bt.shape[1]),
                                   ctypes.c_int(Hkv), ctypes.c_int(d), ctypes.c_int(page))
    return k_out, v_out


def attention(q, k_pool, v_pool, block_table, prefix_len, suffix_len, scale):
    """fp64 output [sum_S, Hq, d] for every suffix row (pools already appended)."""
    q, k_pool, v_pool = _u16(q), _u16(k_pool), _u16(v_pool)
    bt, pl, sl = _i32(block_table), _i32(prefix_len), _i32(suffix_len)
    n, Hq, d = q.shape
    _, Hkv, page, _ = k_pool.shape
    assert n == int(sl.sum()) and Hq % Hkv == 0
    out = np.zeros((n, Hq, d), dtype=np.float64)
    _load().prism_oracle_attention(_p(q), _p(k_pool), _p(v_pool), _p(bt), _p(pl), _p(sl),
                                   ctypes.c_int(bt.shape[0]), ctypes.c_int(bt.shape[1]),
                                   ctypes.c_int(Hq), ctypes.c_int(Hkv), ctypes.c_int(d),
                                   ctypes.c_int(page), ctypes.c_double(scale), _p(out))
    return out


def attention_rows(q, k_pool, v_pool, block_table, prefix_len, suffix_len, scale, rows,
                   want_weights: bool = False):
    """fp64 output [n, d] for the (request, suffix row, q head) triples in rows.
    With want_weights also returns [n, max_T] normalised softmax weights
    (zero beyond each row's visible length)."""
    q, k_pool, v_pool = _u16(q), _u16(k_pool), _u16(v_pool)
    bt, pl, sl = _i32(block_table), _i32(prefix_len), _i32(suffix_len)
    rows = _i32(rows).reshape(-1, 3)
    _, Hq, d = q.shape
    _, Hkv, page, _ = k_pool.shape
    n = rows.shape[0]
    out = np.zeros((n, d), dtype=np.float64)
    wstride = int((pl + sl).max()) if want_weights else 0
    w = np.zeros((n, wstride), dtype=np.float64) if want_weights else None
    _load().prism_oracle_attention_rows(_p(q), _p(k_pool), _p(v_pool), _p(bt), _p(pl), _p(sl),
                                        ctypes.c_int(bt.shape[0]), ctypes.c_int(bt.shape[1]),
                                        ctypes.c_int(Hq), ctypes.c_int(Hkv), ctypes.c_int(d),
                                        ctypes.c_int(page), ctypes.c_double(scale), _p(rows),
                                        ctypes.c_int(n), _p(out),
                                        _p(w) if want_weights else None, ctypes.c_int(wstride))
    return (out, w) if want_weights else out
