"""ctypes binding over libfgattn.so: same names as the C ABI in include/fgattn.h.

Argument marshalling only -- every step of the path runs in the library's HIP kernels.
torch is used for device memory and streams.  There is no fallback: if the library has
not been built, importing a symbol from it raises.
"""
import ctypes
import os

from . import build as _build


class FgattnParams(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("L", ctypes.c_int32), ("d", ctypes.c_int32),
                ("M", ctypes.c_int32), ("N", ctypes.c_int32),
                ("q_stride_b", ctypes.c_int64), ("q_stride_h", ctypes.c_int64), ("q_stride_l", ctypes.c_int64),
                ("k_stride_b", ctypes.c_int64), ("k_stride_h", ctypes.c_int64), ("k_stride_l", ctypes.c_int64),
                ("v_stride_b", ctypes.c_int64), ("v_stride_h", ctypes.c_int64), ("v_stride_l", ctypes.c_int64),
                ("o_stride_b", ctypes.c_int64), ("o_stride_h", ctypes.c_int64), ("o_stride_l", ctypes.c_int64),
                ("scale", ctypes.c_float), ("flags", ctypes.c_int32)]


FLAG_STATIC_ASSIGN, FLAG_FIFO_QUEUE, FLAG_REUSE_PLAN, FLAG_MASK_ROWS_IN_HBM, FLAG_MASK_ONE_TILE_CHUNKS = 1, 2, 4, 8, 16
E_NULL, E_SHAPE, E_STRIDE, E_ALIGN, E_WORKSPACE, E_SCALE, E_DEVICE, E_MASK, E_FLAGS, E_STATIC_LIMIT = range(-1, -11, -1)
STATIC_MAX_ITEMS = 65536

_lib = None


class FgattnError(RuntimeError):
    def __init__(self, code):
        self.code = code
        super().__init__("fgattn error %d: %s" % (code, fgattn_strerror(code)))


def lib():
    """The loaded C-ABI library; raises if it has not been built (there is no CPU fallback)."""
    global _lib
    if _lib is None:
        path = _build.LIBFGATTN
        if not os.path.exists(path):
            raise RuntimeError("libfgattn.so is missing: run __graft_entry__.build() (hipcc, gfx950) first")
        L = ctypes.CDLL(path)
        vp, i64p, pp = ctypes.c_void_p, ctypes.c_void_p, ctypes.POINTER(FgattnParams)
        L.fgattn_workspace_bytes.argtypes = [pp]
        L.fgattn_workspace_bytes.restype = ctypes.c_size_t
        L.fgattn_forward.argtypes = [vp, vp, vp, i64p, vp, pp, vp, vp, vp, ctypes.c_size_t, vp]
        L.fgattn_forward.restype = ctypes.c_int
        L.fgattn_forward_static.argtypes = [vp, vp, vp, i64p, vp, pp, vp, vp, vp]
        L.fgattn_forward_static.restype = ctypes.c_int
        L.fgattn_forward_part.argtypes = [vp, vp, vp, i64p, vp, pp, vp, vp, vp, ctypes.c_size_t, ctypes.c_int, vp]
        L.fgattn_forward_part.restype = ctypes.c_int
        L.fgattn_issue_probe.argtypes = [ctypes.c_int, ctypes.c_int, vp, ctypes.c_size_t, ctypes.POINTER(ctypes.c_double), vp]
        L.fgattn_issue_probe.restype = ctypes.c_int
        L.fgattn_forward_grouped.argtypes = [vp, vp, vp, vp, i64p, vp, vp, pp, vp, vp, vp, ctypes.c_size_t, vp]
        L.fgattn_forward_grouped.restype = ctypes.c_int
        L.fgattn_dense_forward.argtypes = [vp, vp, vp, pp, vp, vp, vp, ctypes.c_size_t, vp]
        L.fgattn_dense_forward.restype = ctypes.c_int
        L.fgattn_plan.argtypes = [i64p, pp, vp, ctypes.c_size_t, vp]
        L.fgattn_plan.restype = ctypes.c_int
        L.fgattn_validate_mask.argtypes = [i64p, vp, pp, vp, ctypes.c_size_t, vp]
        L.fgattn_validate_mask.restype = ctypes.c_int
        L.fgattn_mask_workspace_bytes.argtypes = [pp]
        L.fgattn_mask_workspace_bytes.restype = ctypes.c_size_t
        L.fgattn_mask_select.argtypes = [vp, vp, pp, ctypes.c_float, vp, vp, ctypes.c_size_t, vp]
        L.fgattn_mask_select.restype = ctypes.c_int
        L.fgattn_mask_emit.argtypes = [pp, vp, vp, ctypes.c_int64, vp, ctypes.c_size_t, vp]
        L.fgattn_mask_emit.restype = ctypes.c_int
        L.fgattn_group_workspace_bytes.argtypes = [pp, ctypes.c_int]
        L.fgattn_group_workspace_bytes.restype = ctypes.c_size_t
        L.fgattn_group_select.argtypes = [i64p, vp, pp, ctypes.c_int, vp, vp, vp, ctypes.c_size_t, vp]
        L.fgattn_group_select.restype = ctypes.c_int
        L.fgattn_group_emit.argtypes = [pp, ctypes.c_int, vp, vp, vp, vp, ctypes.c_int64, vp, ctypes.c_size_t, vp]
        L.fgattn_group_emit.restype = ctypes.c_int
        L.fgattn_grid_size.argtypes = [pp]
        L.fgattn_grid_size.restype = ctypes.c_int
        L.fgattn_strerror.argtypes = [ctypes.c_int]
        L.fgattn_strerror.restype = ctypes.c_char_p
        _lib = L
    return _lib


def fgattn_strerror(code):
    return lib().fgattn_strerror(int(code)).decode()


def make_params(q, k, v, out, M, N, scale, flags=0):
    """fgattn_params for [B, H, L, d] tensors (any strides with a contiguous last dim)."""
    B, H, L, d = q.shape
    for t in (q, k, v, out):
        assert t.dim() == 4 and t.stride(3) == 1
    p = FgattnParams(B, H, L, d, M, N,
                     q.stride(0), q.stride(1), q.stride(2), k.stride(0), k.stride(1), k.stride(2),
                     v.stride(0), v.stride(1), v.stride(2), out.stride(0), out.stride(1), out.stride(2),
                     float(scale), int(flags))
    return p


def fgattn_workspace_bytes(params):
    return int(lib().fgattn_workspace_bytes(ctypes.byref(params)))


def _stream_ptr(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _check(rc):
    if rc != 0:
        raise FgattnError(rc)


def fgattn_forward(q, k, v, mask_indptr, mask_indices, params, out, lse, workspace, stream=None):
    """Enqueue the sparse forward pass on `stream` (default: torch's current stream)."""
    _check(lib().fgattn_forward(q.data_ptr(), k.data_ptr(), v.data_ptr(), mask_indptr.data_ptr(),
                                mask_indices.data_ptr(), ctypes.byref(params), out.data_ptr(), lse.data_ptr(),
                                workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                _stream_ptr(stream)))


def fgattn_forward_static(q, k, v, mask_indptr, mask_indices, params, out, lse, stream=None):
    """The sparse forward pass without a workspace argument (scratch inside the library's device image)."""
    _check(lib().fgattn_forward_static(q.data_ptr(), k.data_ptr(), v.data_ptr(), mask_indptr.data_ptr(),
                                       mask_indices.data_ptr(), ctypes.byref(params), out.data_ptr(), lse.data_ptr(),
                                       _stream_ptr(stream)))


PART_GATHER, PART_COMPUTE, PART_GATHER_RING3, PART_GATHER_ONE_WG = 1, 2, 3, 4


def fgattn_forward_grouped(q, k, v, group_tiles, union_indptr, union_indices, union_members, params, out, lse, workspace,
                           stream=None):
    """Sparse forward pass over grouped query tiles (union key lists with per-member masks)."""
    _check(lib().fgattn_forward_grouped(q.data_ptr(), k.data_ptr(), v.data_ptr(), group_tiles.data_ptr(),
                                        union_indptr.data_ptr(), union_indices.data_ptr(), union_members.data_ptr(),
                                        ctypes.byref(params), out.data_ptr(), lse.data_ptr(), workspace.data_ptr(),
                                        workspace.numel() * workspace.element_size(), _stream_ptr(stream)))


def fgattn_forward_part(q, k, v, mask_indptr, mask_indices, params, out, lse, workspace, part, stream=None):
    """Measurement aid: one half of the forward kernel (results in out / lse are meaningless)."""
    _check(lib().fgattn_forward_part(q.data_ptr(), k.data_ptr(), v.data_ptr(), mask_indptr.data_ptr(),
                                     mask_indices.data_ptr(), ctypes.byref(params), out.data_ptr(), lse.data_ptr(),
                                     workspace.data_ptr(), workspace.numel() * workspace.element_size(), int(part),
                                     _stream_ptr(stream)))


def fgattn_issue_probe(other_valu_per_16_mfma, iters, scratch, stream=None):
    """Measurement aid: enqueues the instruction-issue probe; returns the MFMA FLOP count of the launch."""
    flop = ctypes.c_double(0.0)
    _check(lib().fgattn_issue_probe(int(other_valu_per_16_mfma), int(iters), scratch.data_ptr(),
                                    scratch.numel() * scratch.element_size(), ctypes.byref(flop), _stream_ptr(stream)))
    return flop.value


def fgattn_dense_forward(q, k, v, params, out, lse, workspace, stream=None):
    _check(lib().fgattn_dense_forward(q.data_ptr(), k.data_ptr(), v.data_ptr(), ctypes.byref(params),
                                      out.data_ptr(), lse.data_ptr(), workspace.data_ptr(),
                                      workspace.numel() * workspace.element_size(), _stream_ptr(stream)))


def fgattn_mask_workspace_bytes(params):
    return int(lib().fgattn_mask_workspace_bytes(ctypes.byref(params)))


def fgattn_mask_select(q, k, params, top_p, mask_indptr, workspace, stream=None):
    """Top-p mask, first half: fills mask_indptr (device int64) and the per-block cuts in `workspace`."""
    _check(lib().fgattn_mask_select(q.data_ptr(), k.data_ptr(), ctypes.byref(params), float(top_p), mask_indptr.data_ptr(),
                                    workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream_ptr(stream)))


def fgattn_mask_emit(params, mask_indptr, mask_indices, workspace, stream=None):
    """Top-p mask, second half: writes the kept key-block ids (ascending per query block) into mask_indices."""
    _check(lib().fgattn_mask_emit(ctypes.byref(params), mask_indptr.data_ptr(), mask_indices.data_ptr(),
                                  int(mask_indices.numel()), workspace.data_ptr(),
                                  workspace.numel() * workspace.element_size(), _stream_ptr(stream)))


GROUP_CONSECUTIVE, GROUP_XOR = 0, 1


def fgattn_group_workspace_bytes(params, mode):
    return int(lib().fgattn_group_workspace_bytes(ctypes.byref(params), int(mode)))


def fgattn_group_select(mask_indptr, mask_indices, params, mode, group_tiles, union_indptr, workspace, stream=None):
    """Query-tile grouping, first half: fills group_tiles and union_indptr (device tensors)."""
    _check(lib().fgattn_group_select(mask_indptr.data_ptr(), mask_indices.data_ptr(), ctypes.byref(params), int(mode),
                                     group_tiles.data_ptr(), union_indptr.data_ptr(), workspace.data_ptr(),
                                     workspace.numel() * workspace.element_size(), _stream_ptr(stream)))


def fgattn_group_emit(params, mode, group_tiles, union_indptr, union_indices, union_members, workspace, stream=None):
    """Query-tile grouping, second half: fills union_indices / union_members."""
    _check(lib().fgattn_group_emit(ctypes.byref(params), int(mode), group_tiles.data_ptr(), union_indptr.data_ptr(),
                                   union_indices.data_ptr(), union_members.data_ptr(), int(union_indices.numel()),
                                   workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                   _stream_ptr(stream)))


def fgattn_plan(mask_indptr, params, workspace, stream=None):
    _check(lib().fgattn_plan(mask_indptr.data_ptr(), ctypes.byref(params), workspace.data_ptr(),
                             workspace.numel() * workspace.element_size(), _stream_ptr(stream)))


def fgattn_validate_mask(mask_indptr, mask_indices, params, workspace, stream=None):
    """Returns 0 or E_MASK (synchronous)."""
    rc = lib().fgattn_validate_mask(mask_indptr.data_ptr(), mask_indices.data_ptr(), ctypes.byref(params),
                                    workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                    _stream_ptr(stream))
    if rc not in (0, E_MASK):
        raise FgattnError(rc)
    return rc


def fgattn_grid_size(params):
    return int(lib().fgattn_grid_size(ctypes.byref(params)))
