"""ORACLE -- test infrastructure, not product.

Plain fp64 CPU definition of masked (fine-grained sparse) attention, written from the
paper's problem statement (Sec. 2; Sec. 4.1; Fig. 1b).  It shares no code with the HIP
path and is imported only by tests, the smoke check and the benchmark's CPU-baseline leg.

`attention(...)` evaluates chosen work items with the C implementation in
fgattn_oracle.c (built with gcc on first use).  `pool(...)` and `topp_rows(...)` are the
mean-query/key top-p mask of Sec. 4.3 (fgmask_oracle.c).
"""
import ctypes
import os
import subprocess

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(_DIR, "libfgattn_oracle.so")
MASK_LIB = os.path.join(_DIR, "libfgmask_oracle.so")
_lib = None
_mask_lib = None


def build(force=True):
    """Compile the C oracle with gcc (host only)."""
    if force or not os.path.exists(LIB):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", os.path.join(_DIR, "fgattn_oracle.c"), "-o", LIB,
               "-lm"]
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if r.returncode != 0:
            raise RuntimeError("oracle build failed:\n" + r.stdout)
    if force or not os.path.exists(MASK_LIB):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fPIC", "-shared", os.path.join(_DIR, "fgmask_oracle.c"),
               "-o", MASK_LIB, "-lm"]
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if r.returncode != 0:
            raise RuntimeError("mask oracle build failed:\n" + r.stdout)
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


def _load_mask():
    global _mask_lib
    if _mask_lib is None:
        if not os.path.exists(MASK_LIB):
            build()
        lib = ctypes.CDLL(MASK_LIB)
        lib.fgmask_oracle_pool.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                           ctypes.c_void_p]
        lib.fgmask_oracle_pool.restype = None
        lib.fgmask_oracle_row.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_double,
                                          ctypes.c_double, ctypes.c_void_p, ctypes.c_void_p]
        lib.fgmask_oracle_row.restype = ctypes.c_int32
        _mask_lib = lib
    return _mask_lib


def pool(x_bits, rows_per_block):
    """Block means of Sec. 4.3 as bf16 bits: x [..., L, d] -> [slices, ceil(L/rows_per_block), d]."""
    x = np.ascontiguousarray(x_bits, dtype=np.uint16)
    L, d = x.shape[-2], x.shape[-1]
    slices = x.size // (L * d)
    nb = (L + rows_per_block - 1) // rows_per_block
    out = np.empty((slices, nb, d), dtype=np.uint16)
    _load_mask().fgmask_oracle_pool(x.ctypes.data, slices, L, d, int(rows_per_block), out.ctypes.data)
    return out


def topp_rows(q_bits, k_bits, M, N, scale, p, rows=None):
    """Top-p selection of Sec. 4.3 for the given work items (w = slice*ceil(L/M) + i; default all).

    Returns a list of (kept, order, cum) per requested item: `order` ranks all key blocks of the
    item's slice (most probable first, ties by ascending id), `cum` is the cumulative probability
    along it, and the mask keeps order[:kept].
    """
    qp = pool(q_bits, M)
    kp = pool(k_bits, N)
    slices, QB, d = qp.shape
    G = kp.shape[1]
    if rows is None:
        rows = range(slices * QB)
    lib = _load_mask()
    res = []
    for w in rows:
        s, i = divmod(int(w), QB)
        order = np.empty(G, dtype=np.int32)
        cum = np.empty(G, dtype=np.float64)
        qa = np.ascontiguousarray(qp[s, i])
        ka = np.ascontiguousarray(kp[s])
        kept = lib.fgmask_oracle_row(qa.ctypes.data, ka.ctypes.data, G, d, float(scale), float(p), order.ctypes.data,
                                     cum.ctypes.data)
        if kept < 0:
            raise MemoryError("mask oracle allocation failed")
        res.append((int(kept), order, cum))
    return res


def topp_csr(q_bits, k_bits, M, N, scale, p):
    """The whole mask as CSR (ascending key-block ids per item): (indptr int64, indices int32)."""
    rows = topp_rows(q_bits, k_bits, M, N, scale, p)
    indptr = np.zeros(len(rows) + 1, dtype=np.int64)
    parts = []
    for n, (kept, order, _) in enumerate(rows):
        parts.append(np.sort(order[:kept]))
        indptr[n + 1] = indptr[n] + kept
    indices = np.concatenate(parts).astype(np.int32) if parts else np.zeros(0, dtype=np.int32)
    return indptr, indices
