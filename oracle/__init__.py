"""ORACLE -- test infrastructure, not product.

Plain fp64 CPU definition of masked (fine-grained sparse) attention, written from the
paper's problem statement (Sec. 2; Sec. 4.1; Fig. 1b).  It shares no code with the HIP
path and is imported only by tests, the smoke check and the benchmark's CPU-baseline leg.

`attention(...)` evaluates chosen work items with the C implementation in
fgattn_oracle.c (built with gcc on first use).
"""
import ctypes
import os
import subprocess

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(_DIR, "libfgattn_oracle.so")
_lib = None


def build(force=True):
    """Compile the C oracle with gcc (host only)."""
    if force or not os.path.exists(LIB):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", os.path.join(_DIR, "fgattn_oracle.c"), "-o", LIB,
               "-lm"]
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if r.returncode != 0:
            raise RuntimeError("oracle build failed:\n" + r.stdout)
    return LIB


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            build()
        lib = ctypes.CDLL(LIB)
        lib.fgattn_oracle_items.argtypes = [ctypes.c_void_p] * 3 + [ctypes.c_int32] * 5 + [ctypes.c_double] + \
            [ctypes.c_void_p] * 3 + [ctypes.c_int64] + [ctypes.c_void_p] * 2
        lib.fgattn_oracle_items.restype = ctypes.c_int
        lib.fgattn_oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def threads():
    """Host threads the oracle uses (OpenMP's maximum)."""
    return int(_load().fgattn_oracle_threads())


def attention(q_bits, k_bits, v_bits, M, N, scale, indptr, indices, items=None):
    """Masked attention for the given work items.

    q_bits, k_bits, v_bits: uint16 bf16 bit patterns, [..., L, d] contiguous (leading dims
    are folded into slices).  indptr/indices: CSR of active key-group ids per
    (slice, query block).  items: work-item ids (default: all).
    Returns (out [n_items, M, d] float64, lse [n_items, M] float64); rows past L are NaN.
    """
    q = np.ascontiguousarray(q_bits, dtype=np.uint16)
    k = np.ascontiguousarray(k_bits, dtype=np.uint16)
    v = np.ascontiguousarray(v_bits, dtype=np.uint16)
    L, d = q.shape[-2], q.shape[-1]
    slices = q.size // (L * d)
    QB = (L + M - 1) // M
    indptr = np.ascontiguousarray(indptr, dtype=np.int64)
    indices = np.ascontiguousarray(indices, dtype=np.int32)
    assert indptr.shape == (slices * QB + 1,) and indptr[0] == 0 and indptr[-1] == indices.size
    if items is None:
        items = np.arange(slices * QB, dtype=np.int64)
    items = np.ascontiguousarray(items, dtype=np.int64)
    out = np.full((items.size, M, d), np.nan, dtype=np.float64)
    lse = np.full((items.size, M), np.nan, dtype=np.float64)
    rc = _load().fgattn_oracle_items(q.ctypes.data, k.ctypes.data, v.ctypes.data, slices, L, d, M, N, float(scale),
                                     indptr.ctypes.data, indices.ctypes.data if indices.size else None,
                                     items.ctypes.data, items.size, out.ctypes.data, lse.ctypes.data)
    if rc != 0:
        raise ValueError("oracle rejected its input (group id or item id out of range)")
    return out, lse
