"""CPU oracle for top-k selection -- TEST INFRASTRUCTURE ONLY.

This package is the parity reference the GPU library is checked against.  It is
independent of the GPU path: it shares no code with it and neither imports the
other.  Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline``
leg of ``bench.py`` may import it; the product never does.

Contents
--------
``topk_oracle.c``  the definition written out: sort every (element, index) pair
                   of a row with a float-semantic comparator and take the first
                   k (paper Section 1 problem statement; Section 2.3.1, pivot
                   and filter), plus an O(n*k) brute-force selector.
``radix_ref.py``   the paper's Algorithm 1 (countBin / selectBin /
                   selectCandidate / filter, Section 2.3.1) and the adaptive
                   scaling of Section 4.3, step by step in numpy, for checking
                   per-pass internals and the robustness claims.

The functions below are thin ctypes wrappers around the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "topk_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

F32, F16, BF16 = 0, 1, 2
_ELEM = {F32: 4, F16: 2, BF16: 2}

_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain C99, -O2, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-std=c99", "-O2", "-fno-fast-math", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        lib.oracle_decode.restype = ctypes.c_double
        lib.oracle_decode.argtypes = [ci, ctypes.c_uint32]
        lib.oracle_rank_cmp.restype = ci
        lib.oracle_rank_cmp.argtypes = [ci, ctypes.c_uint32, ctypes.c_uint32]
        lib.oracle_sort_row.restype = ci
        lib.oracle_sort_row.argtypes = [vp, ci, i64, ci, vp]
        for name in ("oracle_topk_sort", "oracle_topk_bruteforce"):
            fn = getattr(lib, name)
            fn.restype = ci
            fn.argtypes = [vp, ci, i64, i64, i64, ci, vp, vp]
        _lib = lib
    return _lib


def _as_bits(keys: np.ndarray, dtype: int) -> np.ndarray:
    """Keys as a C-contiguous 2-D array of raw storage words (uint32 / uint16)."""
    want = np.uint32 if dtype == F32 else np.uint16
    a = np.ascontiguousarray(keys)
    if a.dtype == np.float32 and dtype == F32:
        a = a.view(np.uint32)
    elif a.dtype == np.float16 and dtype == F16:
        a = a.view(np.uint16)
    if a.dtype != want:
        raise TypeError("keys must be float32/float16 or raw %s words for dtype %d" % (want.__name__, dtype))
    if a.ndim == 1:
        a = a[None, :]
    if a.ndim != 2:
        raise ValueError("keys must be [n] or [batch, n]")
    return a


def decode(dtype: int, bits: int) -> float:
    """Value of one storage word, as the oracle reads it."""
    return float(_load().oracle_decode(dtype, int(bits)))


def rank_cmp(dtype: int, abits: int, bbits: int) -> int:
    """-1 / 0 / +1: the oracle's preorder on two storage words."""
    return int(_load().oracle_rank_cmp(dtype, int(abits), int(bbits)))


def sort_row(keys: np.ndarray, dtype: int, largest: bool) -> np.ndarray:
    """Full oracle order of ONE row: int64 indices, best element first."""
    a = _as_bits(keys, dtype)
    if a.shape[0] != 1:
        raise ValueError("sort_row takes a single row")
    n = a.shape[1]
    order = np.empty(n, dtype=np.int64)
    rc = _load().oracle_sort_row(a.ctypes.data, dtype, n, int(bool(largest)), order.ctypes.data)
    if rc:
        raise RuntimeError("oracle_sort_row failed with code %d" % rc)
    return order


def _run(fn_name: str, keys, dtype, k, largest):
    a = _as_bits(keys, dtype)
    batch, n = a.shape
    vals = np.empty((batch, k), dtype=a.dtype)
    idx = np.empty((batch, k), dtype=np.int64)
    rc = getattr(_load(), fn_name)(
        a.ctypes.data, dtype, batch, n, int(k), int(bool(largest)), vals.ctypes.data, idx.ctypes.data
    )
    if rc:
        raise RuntimeError("%s failed with code %d" % (fn_name, rc))
    return vals, idx


def topk(keys: np.ndarray, dtype: int, k: int, largest: bool = True):
    """Oracle top-k by full sort.  Returns (value bits [batch,k], int64 indices [batch,k]),
    each row best-first, lowest index first among equal elements."""
    return _run("oracle_topk_sort", keys, dtype, k, largest)


def topk_bruteforce(keys: np.ndarray, dtype: int, k: int, largest: bool = True):
    """Independent O(n*k) selector; same output convention as :func:`topk`."""
    return _run("oracle_topk_bruteforce", keys, dtype, k, largest)
