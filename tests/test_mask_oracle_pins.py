"""Pins for the top-p mask oracle (paper Sec. 4.3): each test fixes it to something other than itself.

The paper prints no worked numeric example, so the pins are: the definition written a
second time in numpy and with torch's library softmax / sort / cumsum, closed forms
(uniform scores, a single dominant key block, hand-computed block means) and invariants
(mass of the kept set, nesting in p).  The mutation test at the end plants mistakes in a
copy of the C source and requires the numpy pin to notice each.
"""
import ctypes
import math
import os
import subprocess

import numpy as np
import pytest
import torch

from paper_2509_16518_amd import workloads as W

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "fgmask_oracle.c")


def rand_bits(rng, shape, lo=-2.0, hi=2.0):
    return W.f32_to_bf16_bits(rng.uniform(lo, hi, size=shape).astype(np.float32))


def numpy_pool(x_bits, rows):
    """Block means the way the reading fixes them: fp32 running sum in row order, fp32 divide, one bf16 rounding."""
    x = W.bf16_bits_to_f64(x_bits).astype(np.float32)
    S, L, d = x.shape
    nb = -(-L // rows)
    out = np.empty((S, nb, d), dtype=np.uint16)
    for b in range(nb):
        blk = x[:, b * rows:min((b + 1) * rows, L), :]
        acc = np.cumsum(blk, axis=1, dtype=np.float32)[:, -1, :]     # sequential fp32 adds
        out[:, b, :] = W.f32_to_bf16_bits((acc / np.float32(blk.shape[1])).astype(np.float32))
    return out


def numpy_topp(qp_bits, kp_bits, scale, p):
    """Sec. 4.3 steps 2-3 on pooled bf16 tensors of one slice: list of kept key-block id arrays per query block."""
    qa = W.bf16_bits_to_f64(qp_bits)
    ka = W.bf16_bits_to_f64(kp_bits)
    s = scale * (qa @ ka.T)
    e = np.exp(s - s.max(axis=1, keepdims=True))
    a = e / e.sum(axis=1, keepdims=True)
    kept = []
    for i in range(a.shape[0]):
        order = np.argsort(-a[i], kind="stable")          # ties: ascending id
        c = np.cumsum(a[i][order])
        n = int(np.searchsorted(c, p, side="left")) + 1   # first position with c >= p
        kept.append(np.sort(order[:min(n, order.size)]))
    return kept


@pytest.mark.parametrize("L,M,N,d", [(48, 4, 2, 16), (50, 8, 3, 8), (33, 16, 1, 32), (40, 1, 1, 8)])
def test_matches_second_numpy_definition(oracle_mod, L, M, N, d):
    rng = np.random.default_rng(L * 100 + M)
    S = 2
    q = rand_bits(rng, (S, L, d), -3, 3)
    k = rand_bits(rng, (S, L, d), -3, 3)
    qp, kp = numpy_pool(q, M), numpy_pool(k, N)
    assert np.array_equal(oracle_mod.pool(q, M), qp) and np.array_equal(oracle_mod.pool(k, N), kp)
    QB = qp.shape[1]
    for p in (0.3, 0.9):
        rows = oracle_mod.topp_rows(q, k, M, N, 0.41, p)
        for s in range(S):
            ref = numpy_topp(qp[s], kp[s], 0.41, p)
            for i in range(QB):
                kept, order, cum = rows[s * QB + i]
                assert np.array_equal(np.sort(order[:kept]), ref[i]), (s, i, p)
                assert abs(cum[-1] - 1.0) < 1e-12 and np.all(np.diff(cum) >= 0)


def test_matches_torch_library_routines(oracle_mod):
    rng = np.random.default_rng(11)
    S, L, d, M, N = 1, 64, 16, 4, 4
    q, k = rand_bits(rng, (S, L, d), -3, 3), rand_bits(rng, (S, L, d), -3, 3)
    qa = torch.from_numpy(W.bf16_bits_to_f64(oracle_mod.pool(q, M)[0]))
    ka = torch.from_numpy(W.bf16_bits_to_f64(oracle_mod.pool(k, N)[0]))
    a = torch.softmax(0.25 * qa @ ka.T, dim=1)
    srt, idx = torch.sort(a, dim=1, descending=True, stable=True)
    cum = torch.cumsum(srt, dim=1)
    rows = oracle_mod.topp_rows(q, k, M, N, 0.25, 0.8)
    for i, (kept, order, c) in enumerate(rows):
        n = int((cum[i] < 0.8).sum().item()) + 1
        assert kept == n
        assert set(order[:kept].tolist()) == set(idx[i, :n].tolist())
        assert np.allclose(c, cum[i].numpy(), atol=1e-12)


def test_pooling_closed_forms(oracle_mod):
    f = lambda a: W.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))
    # mean of 1,2,3,4 = 2.5 exactly; a short last block divides by its own row count: mean(5, 7) = 6
    x = f([1, 2, 3, 4, 5, 7]).reshape(1, 6, 1)
    got = W.bf16_bits_to_f64(oracle_mod.pool(x, 4))
    assert got.reshape(-1).tolist() == [2.5, 6.0]
    # blocks of one row are the rows themselves, bit for bit
    rng = np.random.default_rng(0)
    y = rand_bits(rng, (2, 9, 4))
    assert np.array_equal(oracle_mod.pool(y, 1), y)
    # one rounding, to nearest even: mean(1, 1 + 2^-7) = 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> 1
    z = f([1.0, 1.0 + 2.0 ** -7]).reshape(1, 2, 1)
    assert W.bf16_bits_to_f64(oracle_mod.pool(z, 2)).item() == 1.0
    # the columns are pooled independently
    w = f([[1, 10], [3, 30]]).reshape(1, 2, 2)
    assert W.bf16_bits_to_f64(oracle_mod.pool(w, 2)).reshape(-1).tolist() == [2.0, 20.0]


def _bf16_nearest_even_from_f64(x):
    """One rounding of fp64 values to bf16 bits (nearest, ties to even): the nearest of the three bf16 values around
    the fp32-rounded candidate."""
    c = W.f32_to_bf16_bits(x.astype(np.float32)).astype(np.int64)
    mag, sign = c & 0x7FFF, c & 0x8000
    cands = np.stack([sign | np.maximum(mag - 1, 0), c, sign | (mag + 1)], 0)   # (neighbours in magnitude, same sign)
    err = np.abs(W.bf16_bits_to_f64(cands.astype(np.uint16)) - x[None])
    pick = np.argmin(np.where(err == err.min(0, keepdims=True), cands & 1, 9), 0)
    return np.take_along_axis(cands, pick[None], 0)[0].astype(np.uint16)


@pytest.mark.parametrize("rows", [16, 64, 128])
def test_reading_of_the_means_against_the_exact_mean(oracle_mod, rows):
    # The reading fixes HOW the mean is computed (fp32 running sum in row order, fp32 divide, one rounding) so that
    # its bits do not depend on the implementation.  The plain definition is the exact mean rounded once.  On inputs
    # of the workloads' kind (N(0,1) rounded to bf16) the fp32 sums of up to 128 bf16 values are exact and the two
    # agree on every element; with magnitudes spread over many binades they differ in a few elements per 10^5, by
    # one bf16 ulp.  (The exact sum of bf16 values of bounded exponent range fits fp64.)
    rng = np.random.default_rng(100 + rows)

    def compare(values):
        x = W.f32_to_bf16_bits(values.astype(np.float32))
        got = oracle_mod.pool(x, rows).astype(np.int64)
        xf = W.bf16_bits_to_f64(x).reshape(x.shape[0], -1, rows, x.shape[-1])
        exact = _bf16_nearest_even_from_f64(xf.sum(2) / rows).astype(np.int64)
        return np.abs(got - exact)

    d0 = compare(rng.standard_normal((4, rows * 50, 128)))
    assert d0.max() == 0, "the two readings differ on N(0,1) inputs: %d of %d" % (np.count_nonzero(d0), d0.size)
    wide = rng.standard_normal((4, rows * 100, 128)) * np.exp(3.0 * rng.standard_normal((4, rows * 100, 128)))
    d1 = compare(wide)
    assert d1.max() <= 1 and np.count_nonzero(d1) <= d1.size // 2000, (np.count_nonzero(d1), d1.size)


def test_uniform_scores_keep_lowest_ids(oracle_mod):
    # Q = 0: every key block has probability exactly 1/G; G = 128 and p = 0.75 make the cumulative sums exact
    S, L, d, M, N = 1, 256, 8, 16, 2
    q = np.zeros((S, L, d), dtype=np.uint16)
    k = rand_bits(np.random.default_rng(1), (S, L, d))
    for kept, order, cum in oracle_mod.topp_rows(q, k, M, N, 1.0, 0.75):
        assert kept == 96 and order[:96].tolist() == list(range(96))
        assert cum[95] == 0.75


def test_dominant_key_block_is_kept_alone(oracle_mod):
    S, L, d, M, N = 1, 64, 8, 8, 4
    rng = np.random.default_rng(2)
    q = W.f32_to_bf16_bits(np.ones((S, L, d), dtype=np.float32))
    kf = rng.uniform(-0.1, 0.1, size=(S, L, d)).astype(np.float32)
    kf[0, 5 * N:6 * N, :] = 4.0     # key block 5: score 32 against at most 0.8 for the others
    k = W.f32_to_bf16_bits(kf)
    for kept, order, cum in oracle_mod.topp_rows(q, k, M, N, 1.0, 0.9):
        assert kept == 1 and order[0] == 5 and cum[0] > 0.999


def test_mass_invariants_and_nesting(oracle_mod):
    rng = np.random.default_rng(5)
    S, L, d, M, N = 2, 96, 16, 8, 2
    q, k = rand_bits(rng, (S, L, d), -4, 4), rand_bits(rng, (S, L, d), -4, 4)
    prev = None
    for p in (0.1, 0.5, 0.9, 0.99):
        rows = oracle_mod.topp_rows(q, k, M, N, 0.3, p)
        sets = []
        for kept, order, cum in rows:
            assert cum[kept - 1] >= p and (kept == 1 or cum[kept - 2] < p)   # smallest prefix reaching p
            probs = np.diff(np.concatenate([[0.0], cum]))
            assert np.all(np.diff(probs) <= 1e-15)                           # ranked by probability
            sets.append(set(order[:kept].tolist()))
        if prev is not None:
            assert all(a <= b for a, b in zip(prev, sets))                   # a larger p keeps a superset
        prev = sets


def test_csr_form(oracle_mod):
    rng = np.random.default_rng(6)
    S, L, d, M, N = 2, 40, 8, 8, 4
    q, k = rand_bits(rng, (S, L, d), -4, 4), rand_bits(rng, (S, L, d), -4, 4)
    indptr, indices = oracle_mod.topp_csr(q, k, M, N, 0.5, 0.6)
    rows = oracle_mod.topp_rows(q, k, M, N, 0.5, 0.6)
    assert indptr[0] == 0 and indptr[-1] == indices.size and indptr.size == S * 5 + 1
    for w, (kept, order, _) in enumerate(rows):
        seg = indices[indptr[w]:indptr[w + 1]]
        assert np.all(np.diff(seg) > 0) and set(seg.tolist()) == set(order[:kept].tolist())


MUTATIONS = {
    "divide_by_nominal_rows": ("volatile float mean = acc / (float)(r1 - r0);", "volatile float mean = acc / (float)rows_per_block;"),
    "drop_scale": ("s[j] = scale * dot;", "s[j] = dot;"),
    "ascending_sort": ("if (x->p > y->p) return -1;\n  if (x->p < y->p) return 1;", "if (x->p > y->p) return 1;\n  if (x->p < y->p) return -1;"),
    "strictly_greater_than_p": ("if (kept == G && c >= p) kept = t + 1;", "if (kept == G && c > p + 0.02) kept = t + 1;"),
    "no_normaliser": ("rk[j].p = exp(s[j] - m) / z;", "rk[j].p = exp(s[j] - m);"),
    "key_row_stride": ("bf16_to_f32(k_avg[(int64_t)j * d + c])", "bf16_to_f32(k_avg[(int64_t)j * (d - 1) + c])"),
    "truncating_bf16": ("u += 0x7FFFu + ((u >> 16) & 1u);", "u += 0u;"),
    "ties_by_descending_id": ("return (x->j > y->j) - (x->j < y->j);", "return (x->j < y->j) - (x->j > y->j);"),
}


@pytest.mark.parametrize("name", ["unmodified"] + sorted(MUTATIONS))
def test_pins_catch_planted_mistakes(tmp_path, name):
    text = open(SRC).read()
    if name != "unmodified":
        old, new = MUTATIONS[name]
        assert text.count(old) == 1, "mutation site not found: " + name
        text = text.replace(old, new)
    c = tmp_path / "mut.c"
    c.write_text(text)
    so = str(tmp_path / "mut.so")
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-ffp-contract=off", "-fPIC", "-shared", str(c), "-o", so, "-lm"])
    lib = ctypes.CDLL(so)
    lib.fgmask_oracle_pool.argtypes = [ctypes.c_void_p] + [ctypes.c_int32] * 4 + [ctypes.c_void_p]
    lib.fgmask_oracle_pool.restype = None
    lib.fgmask_oracle_row.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_double,
                                      ctypes.c_double, ctypes.c_void_p, ctypes.c_void_p]
    lib.fgmask_oracle_row.restype = ctypes.c_int32

    rng = np.random.default_rng(9)
    S, L, d, M, N = 1, 50, 8, 8, 3
    q, k = rand_bits(rng, (S, L, d), -3, 3), rand_bits(rng, (S, L, d), -3, 3)
    k[0, 12:15, :] = k[0, 3:6, :]          # key blocks 1 and 4 tie exactly
    QB, G = -(-L // M), -(-L // N)
    qp = np.empty((S, QB, d), np.uint16)
    kp = np.empty((S, G, d), np.uint16)
    lib.fgmask_oracle_pool(q.ctypes.data, S, L, d, M, qp.ctypes.data)
    lib.fgmask_oracle_pool(k.ctypes.data, S, L, d, N, kp.ctypes.data)
    agree = np.array_equal(qp, numpy_pool(q, M)) and np.array_equal(kp, numpy_pool(k, N))
    ref_q, ref_k = numpy_pool(q, M), numpy_pool(k, N)
    for p in (0.35, 0.9):
        ref = numpy_topp(ref_q[0], ref_k[0], 0.6, p)
        for i in range(QB):
            order = np.empty(G, np.int32)
            cum = np.empty(G, np.float64)
            qa, ka = np.ascontiguousarray(qp[0, i]), np.ascontiguousarray(kp[0])
            kept = lib.fgmask_oracle_row(qa.ctypes.data, ka.ctypes.data, G, d, 0.6, p, order.ctypes.data, cum.ctypes.data)
            agree = agree and kept == ref[i].size and np.array_equal(np.sort(order[:kept]), ref[i])
            # the ranking itself, where the two tied blocks must appear in ascending order
            pos = {int(j): t for t, j in enumerate(order)}
            agree = agree and pos[1] < pos[4] and abs(cum[-1] - 1.0) < 1e-9
    if name == "unmodified":
        assert agree
    else:
        assert not agree, "pins did not notice mutation " + name
