"""Checks that the pins have teeth: planted mistakes in a COPY of the oracle (CPU only) must be caught.

Each mutation is a textual edit of fgattn_oracle.c compiled into a temporary library; the
brute-force pin (full score matrix in numpy) has to disagree with every mutant.
"""
import ctypes
import os
import subprocess

import numpy as np
import pytest

from paper_2509_16518_amd import workloads as W
from test_oracle_pins import blocks_to_rows, brute_force, key_level_bool_mask, rand_bits, random_csr

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "fgattn_oracle.c")

MUTATIONS = {
    "drop_scale": ("s[a] = scale * dot;", "s[a] = dot;"),
    "value_uses_key_rows": ("const uint16_t* vr = Vb + keys[a] * d;", "const uint16_t* vr = Kb + keys[a] * d;"),
    "wrong_sign_in_exp": ("double p = exp(s[a] - l);", "double p = exp(l - s[a]);"),
    "group_stride_off_by_one": ("for (int64_t key = g * N; key < (g + 1) * N && key < L; key++)",
                                "for (int64_t key = g * N + 1; key < (g + 1) * N + 1 && key < L; key++)"),
    "lse_without_max": ("double l = m + log(sum);", "double l = log(sum);"),
    "block_start_off": ("for (int64_t r = i * M; r < (i + 1) * M && r < L; r++) {\n          const uint16_t* qr = q + (sl * (int64_t)L + r) * d;",
                        "for (int64_t r = i * M; r < (i + 1) * M && r < L; r++) {\n          const uint16_t* qr = q + (sl * (int64_t)L + i * M) * d;"),
    "slice_ignored_for_keys": ("const uint16_t* Kb = k + sl * (int64_t)L * d;", "const uint16_t* Kb = k;"),
}


def run_lib(path, q, k, v, M, N, scale, indptr, indices):
    lib = ctypes.CDLL(path)
    lib.fgattn_oracle_items.argtypes = [ctypes.c_void_p] * 3 + [ctypes.c_int32] * 5 + [ctypes.c_double] + \
        [ctypes.c_void_p] * 3 + [ctypes.c_int64] + [ctypes.c_void_p] * 2
    S, L, d = q.shape
    n = indptr.size - 1
    items = np.arange(n, dtype=np.int64)
    out = np.full((n, M, d), np.nan)
    lse = np.full((n, M), np.nan)
    rc = lib.fgattn_oracle_items(q.ctypes.data, k.ctypes.data, v.ctypes.data, S, L, d, M, N, scale, indptr.ctypes.data,
                                 indices.ctypes.data, items.ctypes.data, n, out.ctypes.data, lse.ctypes.data)
    assert rc == 0
    return out, lse


@pytest.mark.parametrize("name", ["unmodified"] + sorted(MUTATIONS))
def test_pin_catches_planted_mistake(tmp_path, name):
    text = open(SRC).read()
    if name != "unmodified":
        old, new = MUTATIONS[name]
        assert text.count(old) == 1, "mutation site not found: " + name
        text = text.replace(old, new)
    c = tmp_path / "mut.c"
    c.write_text(text)
    so = str(tmp_path / "mut.so")
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", str(c), "-o", so, "-lm"])
    rng = np.random.default_rng(3)
    S, L, d, M, N = 2, 30, 16, 8, 3
    q, k, v = (rand_bits(rng, (S, L, d)) for _ in range(3))
    indptr, indices = random_csr(rng, S, L, M, N, 0.4)
    out, lse = run_lib(so, q, k, v, M, N, 0.37, indptr, indices)
    o, l = blocks_to_rows(out, lse, S, L, M)
    ro, rl = brute_force(q, k, v, 0.37, key_level_bool_mask(L, M, N, indptr, indices, S))
    err = max(np.nanmax(np.abs(o - ro)), np.nanmax(np.abs(l - rl)))
    if name == "unmodified":
        assert err < 1e-12
    else:
        assert not (err < 1e-6), "pin did not notice mutation " + name
