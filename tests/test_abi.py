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
    for field, bad in (("d", 96), ("M", 24), ("N", 0), ("L", 0), ("H", 0), ("flags", 16)):
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
