"""CPU-only checks of the boundary: the library loads, exports every symbol the header declares, and
rejects bad arguments before touching a device."""
import ctypes
import os
import re

import pytest

from paper_2509_16518_amd import build
from paper_2509_16518_amd import fgattn as F

REPO = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(build.LIBFGATTN):
        build.build_hip()
    return F.lib()


def declared_symbols():
    text = open(os.path.join(REPO, "include", "fgattn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fgattn_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = declared_symbols()
    assert {"fgattn_forward", "fgattn_dense_forward", "fgattn_plan", "fgattn_workspace_bytes", "fgattn_validate_mask",
            "fgattn_grid_size", "fgattn_strerror"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_params_struct_matches_header_layout():
    # 6 int32, 12 int64, float, int32 -> 24 + 96 + 8 bytes, no padding surprises
    assert ctypes.sizeof(F.FgattnParams) == 128
    assert F.FgattnParams.q_stride_b.offset == 24 and F.FgattnParams.scale.offset == 120


def test_workspace_bytes_and_shape_validation(lib):
    p = F.FgattnParams(1, 12, 32760, 128, 64, 1, *([0] * 12), 0.1, 0)
    n = lib.fgattn_workspace_bytes(ctypes.byref(p))
    assert n >= 256 + 4 * 12 * 512 and n % 256 == 0
    for field, bad in (("d", 96), ("M", 24), ("N", 0), ("L", 0), ("H", 0), ("flags", 32)):
        q = F.FgattnParams(1, 12, 32760, 128, 64, 1, *([0] * 12), 0.1, 0)
        setattr(q, field, bad)
        assert lib.fgattn_workspace_bytes(ctypes.byref(q)) == 0, field
    assert lib.fgattn_workspace_bytes(None) == 0


def test_null_and_shape_errors_need_no_device(lib):
    assert lib.fgattn_forward(None, None, None, None, None, None, None, None, None, 0, None) == F.E_NULL
    p = F.FgattnParams(1, 1, 64, 128, 64, 1, *([0] * 12), 0.1, 0)
    one = ctypes.c_void_p(4096)   # never dereferenced: argument checks fail first
    p.d = 100
    assert lib.fgattn_forward(one, one, one, one, one, ctypes.byref(p), one, one, one, 1 << 20, None) == F.E_SHAPE
    p.d = 128
    assert lib.fgattn_forward(one, one, one, one, one, ctypes.byref(p), one, one, one, 1 << 20, None) == F.E_STRIDE
    for code in range(0, -10, -1):
        assert lib.fgattn_strerror(code) and b"unknown fgattn" not in lib.fgattn_strerror(code)
    assert b"unknown" in lib.fgattn_strerror(-99)


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    monkeypatch.setattr(F, "_lib", None)
    monkeypatch.setattr(build, "LIBFGATTN", str(tmp_path / "missing.so"))
    with pytest.raises(RuntimeError, match="libfgattn.so is missing"):
        F.lib()


def test_gather_offset_bound_includes_the_bias(lib):
    # K/V rows are addressed with 32-bit byte offsets that also carry a +4096 bias: a slice whose last row ends
    # within 4 KiB below 4 GiB must be rejected, one just under the bound accepted (it then fails on the
    # zero-sized workspace, before any device is touched)
    one = ctypes.c_void_p(4096)
    d, L = 128, 257
    stride = 8388600                      # elements; 2 * stride < 2^24
    assert (L - 1) * stride * 2 + 2 * d <= 0xffffffff < (L - 1) * stride * 2 + 2 * d + 4096

    def call(k_stride, v_stride):
        p = F.FgattnParams(1, 1, L, d, 64, 1, 0, 0, d, 0, 0, k_stride, 0, 0, v_stride, 0, 0, d, 0.1, 0)
        return lib.fgattn_forward(one, one, one, one, one, ctypes.byref(p), one, one, one, 0, None)
    assert call(stride, d) == F.E_STRIDE
    assert call(d, stride) == F.E_STRIDE
    inside = stride - 16                  # 256 rows * 32 bytes less: 8 KiB below the bound
    assert (L - 1) * inside * 2 + 2 * d + 4096 <= 0xffffffff
    assert call(inside, inside) == F.E_WORKSPACE
    assert call(d, d) == F.E_WORKSPACE


def test_dense_call_ignores_n(lib):
    one = ctypes.c_void_p(4096)
    for n in (0, -3, 7):
        p = F.FgattnParams(1, 1, 256, 128, 64, n, 0, 0, 128, 0, 0, 128, 0, 0, 128, 0, 0, 128, 0.1, 0)
        assert lib.fgattn_dense_forward(one, one, one, ctypes.byref(p), one, one, one, 0, None) == F.E_WORKSPACE
    assert lib.fgattn_dense_forward(one, one, one, None, one, one, one, 0, None) == F.E_NULL


def test_build_rejects_a_foreign_m0_write(tmp_path):
    good = tmp_path / "good.s"
    good.write_text("\ts_mov_b32 m0, s5 ; fg_m0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 v1, s[2:3]\n\t; a comment naming m0\n")
    build.check_m0_writes(str(good))
    bad = tmp_path / "bad.s"
    bad.write_text("\ts_mov_b32 m0, s5 ; fg_m0\n\ts_mov_b32 m0, s9\n")
    with pytest.raises(RuntimeError, match="M0 is touched"):
        build.check_m0_writes(str(bad))


def test_build_rejects_a_scalar_base_written_too_close_to_a_gather(tmp_path):
    # a vector-ALU write of a scalar register needs five wait states before a vector-memory instruction reads it; the
    # compiler pads its own instructions but not the ones inside asm statements
    far = tmp_path / "far.s"
    far.write_text("\tv_readfirstlane_b32 s4, v1\n\ts_nop 4\n\tglobal_load_lds_dwordx4 v2, s[4:5]\n"
                   "\tv_readfirstlane_b32 s8, v1\n\ts_mov_b32 m0, s9 ; fg_m0\n\tglobal_load_lds_dwordx4 v2, s[4:5] offset:1024\n")
    build.check_inline_asm_hazards(str(far))
    near = tmp_path / "near.s"
    near.write_text("\tv_readfirstlane_b32 s5, v1\n\ts_mov_b32 m0, s9 ; fg_m0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 v2, s[4:5]\n")
    with pytest.raises(RuntimeError, match="wait states ahead"):
        build.check_inline_asm_hazards(str(near))
    pair = tmp_path / "pair.s"
    pair.write_text("\tv_cmp_lt_f32_e64 s[6:7], v1, v2\n\tv_mov_b32_e32 v3, v4\n\tglobal_load_dword v5, v6, s[6:7]\n")
    with pytest.raises(RuntimeError, match="wait states ahead"):
        build.check_inline_asm_hazards(str(pair))


def test_mask_workspace_is_bounded(lib):
    # the fp32 scores pass through a buffer of at most 1 GiB (whole tiles of 128 query blocks); what grows with the
    # problem is one bit per pair of query block and key block, the block means and 20 bytes per query block
    lib.fgattn_mask_workspace_bytes.restype = ctypes.c_size_t
    def nbytes(H, L, M, flags=0):
        p = F.FgattnParams(1, H, L, 128, M, 1, *([0] * 12), 0.1, flags)
        return lib.fgattn_mask_workspace_bytes(ctypes.byref(p))
    def small_parts(H, L, M):
        rows, G = H * -(-L // M), L
        return rows * 128 * 2 + rows * 20 + rows * -(-G // 32) * 4
    GiB = 1 << 30
    wan, hun = nbytes(12, 32760, 64), nbytes(24, 118800, 128)
    assert 12 * 512 * 32768 * 4 <= wan <= 12 * 512 * 32768 * 4 + small_parts(12, 32760, 64) + 4096    # one chunk: all scores
    assert hun <= GiB + small_parts(24, 118800, 128) + 4096 and hun >= GiB - 128 * 118816 * 4
    one_tile = nbytes(24, 118800, 128, F.FLAG_MASK_ONE_TILE_CHUNKS)
    assert 128 * 118816 * 4 <= one_tile <= 128 * 118816 * 4 + small_parts(24, 118800, 128) + 4096
