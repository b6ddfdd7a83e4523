"""ctypes front end of the C form of the oracle (decode_attention.c).

TEST INFRASTRUCTURE ONLY.  Marshals numpy arrays to the plain-C loops; holds no
arithmetic of its own.  `build()` compiles the C file with gcc next to it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "decode_attention.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle (gcc, -O2, OpenMP).  Returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", _SRC, "-o", tmp, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        p = ctypes.c_void_p
        i = ctypes.c_int
        lib.oracle_half_to_double.restype = ctypes.c_double
        lib.oracle_half_to_double.argtypes = [ctypes.c_uint16]
        lib.oracle_decode.restype = ctypes.c_long
        lib.oracle_decode.argtypes = [p, p, p, p, p, i, i, i, i, i, i, i,
                                      ctypes.c_float, p, p, i, i, i]
        lib.oracle_kv_append.restype = None
        lib.oracle_kv_append.argtypes = [p, p, p, p, p, p, i, i, i, i, i, i]
        _lib = lib
    return _lib


def _ptr(a):
    return None if a is None else ctypes.c_void_p(a.ctypes.data)


def _f16(a):
    assert a.dtype == np.float16 and a.flags["C_CONTIGUOUS"]
    return a


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def half_to_double(bits: int) -> float:
    return _load().oracle_half_to_double(int(bits))


def _geometry(cache, page_table):
    if page_table is None:
        return int(cache.shape[2]), 0, 0
    return 0, int(cache.shape[2]), int(page_table.shape[1])


def decode(q, k_cache, v_cache, seq_lens, scale, page_table=None,
           pair_stride=1, pair_offset=0, nthreads=1):
    """Same contract as decode_attention.decode; rows of skipped pairs are NaN."""
    B, Hq, D = q.shape
    Hkv = k_cache.shape[1]
    assert Hq % Hkv == 0
    sl, pt = _i32(seq_lens), _i32(page_table)
    cap, ps, mp = _geometry(k_cache, pt)
    out = np.full((B, Hq, D), np.nan, dtype=np.float64)
    lse = np.full((B, Hq), np.nan, dtype=np.float64)
    _load().oracle_decode(_ptr(_f16(q)), _ptr(_f16(k_cache)), _ptr(_f16(v_cache)), _ptr(sl),
                          _ptr(pt), B, Hq, Hkv, D, cap, ps, mp, float(np.float32(scale)),
                          _ptr(out), _ptr(lse), int(pair_stride), int(pair_offset), int(nthreads))
    return out, lse


def kv_append(k_cache, v_cache, k_new, v_new, seq_lens, page_table=None) -> None:
    B, Hkv, D = k_new.shape
    sl, pt = _i32(seq_lens), _i32(page_table)
    cap, ps, mp = _geometry(k_cache, pt)
    _load().oracle_kv_append(_ptr(_f16(k_cache)), _ptr(_f16(v_cache)), _ptr(_f16(k_new)),
                             _ptr(_f16(v_new)), _ptr(sl), _ptr(pt), B, Hkv, D, cap, ps, mp)
