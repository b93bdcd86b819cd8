"""Seeded synthetic workloads: bf16 N(0,1) tensors and CSR masks of active key groups.

Input generation only -- no attention arithmetic lives here.  The numbers come from the
counter-based generator in fgw_gen.c (gcc, OpenMP), loaded through ctypes; arrays are
numpy on the host.  The named configurations mirror the video-shaped workloads the
kernel is measured on (locality window on a T x H x W token grid plus random fill; the
micro-benchmark's pure-random masks of paper Sec. 5.1; the skewed list lengths of the
paper's scheduler ablation).
"""
import ctypes
import os
from dataclasses import dataclass, field, replace

import numpy as np

from .. import build as _build

MASK_WINDOW_FILL, MASK_RANDOM, MASK_ALL, MASK_SKEW_HEADS, MASK_SKEW_LEN = range(5)


class _Spec(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("heads", ctypes.c_int32), ("L", ctypes.c_int32), ("M", ctypes.c_int32),
                ("N", ctypes.c_int32), ("gt", ctypes.c_int32), ("gh", ctypes.c_int32), ("gw", ctypes.c_int32),
                ("dt", ctypes.c_int32), ("dh", ctypes.c_int32), ("dw", ctypes.c_int32), ("density", ctypes.c_double),
                ("sigma", ctypes.c_double), ("skew", ctypes.c_double), ("seed", ctypes.c_uint64)]


_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.LIBFGW
        if not os.path.exists(path):
            _build.build_workloads()
        lib = ctypes.CDLL(path)
        lib.fgw_normal_bf16.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_int64]
        lib.fgw_normal_bf16.restype = None
        lib.fgw_mask_count.argtypes = [ctypes.POINTER(_Spec), ctypes.c_void_p]
        lib.fgw_mask_count.restype = ctypes.c_int64
        lib.fgw_mask_fill.argtypes = [ctypes.POINTER(_Spec), ctypes.c_void_p, ctypes.c_void_p]
        lib.fgw_mask_fill.restype = ctypes.c_int
        _lib = lib
    return _lib


@dataclass(frozen=True)
class Workload:
    """One attention problem: shapes, block sizes and the mask recipe."""
    name: str
    H: int                      # heads (batch folded in: B * H slices)
    L: int                      # tokens
    d: int                      # head dim
    M: int                      # query-block rows
    N: int                      # keys per key group
    grid: tuple = (1, 1, 1)     # token grid (T, Hg, Wg); product == L for window masks
    window: tuple = (0, 0, 0)   # window half-widths (dt, dh, dw)
    kind: int = MASK_WINDOW_FILL
    density: float = 0.30
    sigma: float = 0.6
    skew: float = 0.0
    seed: int = 1000
    B: int = 1

    @property
    def scale(self):
        return 1.0 / float(np.sqrt(self.d))

    @property
    def QB(self):
        return (self.L + self.M - 1) // self.M

    @property
    def G(self):
        return (self.L + self.N - 1) // self.N

    @property
    def items(self):
        return self.B * self.H * self.QB


def normal_bf16(seed, stream, shape):
    """bf16 bit patterns (uint16) of N(0,1) draws; a pure function of (seed, stream, index)."""
    out = np.empty(shape, dtype=np.uint16)
    _load().fgw_normal_bf16(seed, stream, out.ctypes.data, out.size)
    return out


def make_qkv(w):
    """Q, K, V as uint16 bf16 bit patterns, each [B, H, L, d] contiguous."""
    shape = (w.B, w.H, w.L, w.d)
    return tuple(normal_bf16(w.seed, s, shape) for s in (1, 2, 3))


def make_qk_local(w, gain=1.0, bandwidth=0.35):
    """Q and K whose scores are local in space-time, as video-DiT attention is (Sec. 4.3): the N(0,1) draws of
    make_qkv plus `gain` times seeded random Fourier features of the token's (t, h, w) grid position, so that
    <q, k> grows towards tokens that are close on the grid.  Returns bf16 bit patterns (q, k), [B, H, L, d]."""
    q, k, _ = make_qkv(w)
    T, Hg, Wg = w.grid
    assert T * Hg * Wg == w.L, "needs a token grid"
    idx = np.arange(w.L)
    pos = np.stack([idx // (Hg * Wg), (idx // Wg) % Hg, idx % Wg], axis=1).astype(np.float64)
    rng = np.random.default_rng(w.seed + 77)
    xq, xk = bf16_bits_to_f64(q), bf16_bits_to_f64(k)
    for h in range(w.H):
        freq = rng.normal(0.0, bandwidth, size=(3, w.d // 2))      # one draw per head, shared by Q and K
        ang = pos @ freq
        feat = gain * np.concatenate([np.cos(ang), np.sin(ang)], axis=1)   # <feat(a), feat(b)> = gain^2 sum cos(freq.(a-b))
        xq[:, h] += feat
        xk[:, h] += feat
    return f32_to_bf16_bits(xq.astype(np.float32)), f32_to_bf16_bits(xk.astype(np.float32))


def make_mask(w):
    """CSR mask: indptr int64 [items + 1], indices int32 [nnz] (ascending key-group ids per item)."""
    spec = _Spec(w.kind, w.B * w.H, w.L, w.M, w.N, w.grid[0], w.grid[1], w.grid[2], w.window[0], w.window[1],
                 w.window[2], w.density, w.sigma, w.skew, w.seed)
    lib = _load()
    indptr = np.zeros(w.items + 1, dtype=np.int64)
    nnz = lib.fgw_mask_count(ctypes.byref(spec), indptr.ctypes.data)
    if nnz < 0:
        raise ValueError("bad mask spec for workload %s" % w.name)
    indices = np.empty(nnz, dtype=np.int32)
    if lib.fgw_mask_fill(ctypes.byref(spec), indptr.ctypes.data, indices.ctypes.data) != 0:
        raise RuntimeError("mask generation failed for workload %s" % w.name)
    return indptr, indices


def bf16_bits_to_f64(bits):
    """Exact widening of bf16 bit patterns to float64 (a bf16 is the top half of an fp32)."""
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def f32_to_bf16_bits(x):
    """Round-to-nearest-even fp32 -> bf16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def active_keys_per_item(w, indptr, indices):
    """Number of keys (not groups) each work item attends: N per active group, fewer for a short last group."""
    keys = np.diff(indptr).astype(np.int64) * w.N
    short = w.G * w.N - w.L
    if short:
        has_last = np.zeros(w.items, dtype=bool)
        pos = np.flatnonzero(indices == w.G - 1)
        has_last[np.searchsorted(indptr, pos, side="right") - 1] = True
        keys -= short * has_last
    return keys


def useful_flop(w, indptr, indices):
    """4*d FLOP per (query row, active key): 2*d for QK^T and 2*d for PV (the rho*N^2*D count of paper Sec. 3)."""
    rows = np.minimum(w.M, w.L - (np.arange(w.items) % w.QB) * w.M)
    return float(np.sum(rows * active_keys_per_item(w, indptr, indices)) * 4.0 * w.d)


def dense_flop(w):
    return 4.0 * w.d * float(w.L) * float(w.L) * w.B * w.H


# ---- named configurations -----------------------------------------------------------------------

TINY = Workload("tiny", H=2, L=1024, d=64, M=16, N=1, grid=(4, 16, 16), window=(1, 3, 3), density=0.30, seed=1001)
WAN_1_3B = Workload("wan-1.3b", H=12, L=32760, d=128, M=64, N=1, grid=(21, 30, 52), window=(2, 4, 4),
                    density=0.30, seed=1002)
HUNYUAN = Workload("hunyuan", H=24, L=118800, d=128, M=128, N=1, grid=(33, 45, 80), window=(2, 6, 6),
                   density=0.20, seed=1004)
WAN_14B_SKEW = Workload("wan-14b-skew", H=40, L=32760, d=128, M=64, N=8, grid=(21, 30, 52), window=(2, 4, 4),
                        kind=MASK_SKEW_HEADS, density=0.30, sigma=0.6, seed=1005)


def sweep(M, N, kind=MASK_WINDOW_FILL, density=0.30):
    """Tile-granularity sweep point on the Tiny shape."""
    tag = {MASK_WINDOW_FILL: "win", MASK_RANDOM: "rnd", MASK_ALL: "all"}[kind]
    return replace(TINY, name="sweep-%s-M%d-N%d" % (tag, M, N), M=M, N=N, kind=kind, density=density, seed=1003)


def dense_of(w):
    """Same shape with every key group active (0% sparsity)."""
    return replace(w, name=w.name + "-all", kind=MASK_ALL)
