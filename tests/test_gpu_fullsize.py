"""Full-size configurations in the launch shape the benchmark times.

The oracle cannot evaluate these in full, so each config is checked two ways:
  * oracle parity on a seeded sample of work items (first block, last partial block, the longest
    and shortest lists, one item per head, random ones; >= 96 items);
  * a closed form that pins the gathered key SET of every row at full scale through the LSE:
    K holds hashed 0/1 entries, query row r is the unit vector e_(r mod d) and scale = ln 2, so
    exp(score) is 1 or 2 and  lse_r = ln(|A| + #{k in A : K[k][r mod d] = 1}).  A dropped, duplicated
    or wrong key changes that integer by >= 1, i.e. the lse by >= 1/(2|A|) ~ 2e-5..1e-4, far above fp32
    rounding -- the random-input tolerance (2e-2) could never see it;
  * a second closed form that pins the gathered VALUE rows of every block of every head (one_hot_value_check):
    every key belongs to one of 8 classes and one of d columns (seeded draws); its K row holds ones in the
    columns of its class, its V row is the unit vector of its column; query row r is the unit vector e_(r mod d)
    and the scale is 64, so a row attends (up to exp(-64)) exactly to the active keys of class (r mod 8) with
    p = 1, all sums are small exact integers in fp32, and  out[r][c] = #{active keys of that class in column c} /
    #{active keys of that class}.  The counts are kept below 128 so that one wrong, dropped or duplicated V
    row moves some output by more than a bf16 ulp; the expected value is checked to half an ulp.
"""
import math

import numpy as np
import pytest
import scipy.sparse as sp
import torch

from paper_2509_16518_amd import workloads as W
from gpu_util import Problem, check_against_oracle, sample_items, say

pytestmark = pytest.mark.gpu


def bit_count_check(w, indptr, indices, heads, what):
    """Runs the LSE closed form on the given heads (all query rows of those heads)."""
    k_bits01 = (W.normal_bf16(w.seed + 77, 5, (w.B, w.H, w.L, w.d)) >> 15).astype(np.uint16)   # hashed 0/1
    kb = (k_bits01 * np.uint16(0x3F80)).astype(np.uint16)                                         # bf16 0.0 / 1.0
    q = np.zeros((w.B, w.H, w.L, w.d), dtype=np.uint16)
    r = np.arange(w.L)
    q[:, :, r, r % w.d] = 0x3F80
    v = W.normal_bf16(w.seed, 3, (w.B, w.H, w.L, w.d))
    prob = Problem(w, q, kb, v, mask=(indptr, indices))
    say("  %s: closed-form run" % what)
    out, lse = prob.run(scale=math.log(2.0))
    assert np.isfinite(out).all()
    worst = 0.0
    for h in heads:
        lo, hi = h * w.QB, (h + 1) * w.QB
        ip = indptr[lo:hi + 1] - indptr[lo]
        ix = indices[indptr[lo]:indptr[hi]]
        A = sp.csr_matrix((np.ones(ix.size, dtype=np.float32), ix, ip), shape=(w.QB, w.G))
        kh = k_bits01[0, h].astype(np.float32)
        assert w.L % w.N == 0
        kg = kh.reshape(w.G, w.N, w.d).sum(axis=1)                    # ones per key group and column
        n1 = np.asarray(A @ kg)                                       # [QB, d] exact small integers
        cnt = np.diff(ip).astype(np.float64) * w.N                    # |A| per block
        rows = np.arange(w.L)
        expect = np.log(cnt[rows // w.M] + n1[rows // w.M, rows % w.d])
        err = np.abs(lse[0, h] - expect)
        worst = max(worst, float(err.max()))
        min_signal = 1.0 / (2.0 * cnt.max() + 1.0)
        assert err.max() < 0.25 * min_signal, (what, h, float(err.max()), min_signal)
    say("  %s: closed-form lse max err %.2e on heads %s" % (what, worst, list(heads)))


def one_hot_value_check(w, indptr, indices, what, classes=8, scale=64.0):
    """Pins the V rows each block gathers, on every block of every head (see the module docstring)."""
    rng = np.random.default_rng(w.seed + 4242)
    S = w.B * w.H
    cls = rng.integers(0, classes, size=(S, w.L), dtype=np.int32)
    col = rng.integers(0, w.d, size=(S, w.L), dtype=np.int32)
    one = np.uint16(0x3F80)
    kb = ((np.arange(w.d, dtype=np.int32) % classes)[None, None, :] == cls[:, :, None]).astype(np.uint16) * one
    vb = np.zeros((S, w.L, w.d), dtype=np.uint16)
    vb[np.arange(S)[:, None], np.arange(w.L)[None, :], col] = one
    q = np.zeros((S, w.L, w.d), dtype=np.uint16)
    r = np.arange(w.L)
    q[:, r, r % w.d] = one
    shape = (w.B, w.H, w.L, w.d)
    prob = Problem(w, q.reshape(shape), kb.reshape(shape), vb.reshape(shape), mask=(indptr, indices))
    del kb, vb, q
    say("  %s: one-hot value closed form, all %d slices" % (what, S))
    out, lse = prob.run(scale=scale)
    del prob
    torch.cuda.empty_cache()
    out = out.reshape(S, w.L, w.d)
    lse = lse.reshape(S, w.L)
    assert np.isfinite(out).all()
    worst_ulp, worst_lse, max_count, sensitive, total = 0.0, 0.0, 0, 0, 0
    rows = np.arange(w.L)
    blk = rows // w.M
    assert w.L % w.N == 0
    for s in range(S):
        lo, hi = s * w.QB, (s + 1) * w.QB
        ip = indptr[lo:hi + 1] - indptr[lo]
        ix = indices[indptr[lo]:indptr[hi]]
        A = sp.csr_matrix((np.ones(ix.size, dtype=np.float32), ix, ip), shape=(w.QB, w.G))
        # per key group: how many of its keys fall on (class, column)
        code = (cls[s] * w.d + col[s]).astype(np.int64)
        F = sp.csr_matrix((np.ones(w.L, dtype=np.float32), (np.arange(w.L) // w.N, code)), shape=(w.G, classes * w.d))
        cnt = np.asarray((A @ F).todense(), dtype=np.float64).reshape(w.QB, classes, w.d)   # exact small integers
        tot = cnt.sum(axis=2)                                                               # keys of the class per block
        c_r = rows % w.d % classes
        num = cnt[blk, c_r]                         # [L, d]
        den = tot[blk, c_r]                         # [L]
        ok = den > 0                                # (a block without a key of the row's class attends to all keys: skipped)
        expect = num[ok] / den[ok][:, None]
        got = out[s][ok]
        with np.errstate(divide="ignore"):
            ulp = np.where(expect > 0, np.exp2(np.floor(np.log2(np.where(expect > 0, expect, 1.0))) - 7.0), 0.0)
        err = np.abs(got - expect)
        tol = 0.5 * ulp * (1.0 + 2.0 ** -6) + 1e-12
        bad = err > tol
        assert not bad.any(), (what, s, int(bad.sum()), float(err[bad].max()))
        worst_ulp = max(worst_ulp, float((err / np.maximum(ulp, 1e-30))[expect > 0].max()))
        el = np.abs(lse[s][ok] - (scale + np.log(den[ok])))
        worst_lse = max(worst_lse, float(el.max()))
        # (fp32 rounding of an lse near 64 + ln(count) is ~4e-6; one key more or less moves it by >= 1 / (2 count))
        assert el.max() < max(0.25 / (2.0 * den.max() + 1.0), 1e-5), (what, s, float(el.max()))
        max_count = max(max_count, int(num.max()))
        sensitive += int((num[ok] < 128).sum())
        total += int(num[ok].size)
    say("  %s: value closed form: worst error %.3f bf16 ulp (bar 0.5), lse max err %.2e, largest count %d, "
        "%.4f%% of the outputs have a count below 128" % (what, worst_ulp, worst_lse, max_count, 100.0 * sensitive / total))
    assert sensitive == total, "a count reached 128: one wrong value row would hide inside a bf16 ulp there"


def run_config(oracle_mod, w, n_random, closed_form_heads):
    say("config %s: generating inputs" % w.name)
    prob = Problem(w)
    say("  nnz %d (density %.4f); sparse forward" % (prob.indices.size, prob.indices.size / (w.items * w.G)))
    got = prob.run()
    items = sample_items(w, prob.indptr, n_random)
    say("  oracle on %d sampled work items" % items.size)
    check_against_oracle(oracle_mod, prob, got, items=items, what=w.name)
    indptr, indices = prob.indptr, prob.indices
    del prob
    torch.cuda.empty_cache()
    bit_count_check(w, indptr, indices, closed_form_heads, w.name)
    one_hot_value_check(w, indptr, indices, w.name)


def test_wan_1_3b_shaped(oracle_mod):
    """H=12, L=32760, d=128, M=64, N=1, 70% sparsity; the final query block has 56 rows."""
    w = W.WAN_1_3B
    assert w.L % w.M == 56
    run_config(oracle_mod, w, n_random=96, closed_form_heads=range(w.H))


def test_wan_14b_shaped_skew(oracle_mod):
    """H=40, M=64, N=8, per-head lognormal density: the load-imbalance stress for the scheduler."""
    w = W.WAN_14B_SKEW
    run_config(oracle_mod, w, n_random=64, closed_form_heads=range(0, w.H, 3))


def test_hunyuan_shaped(oracle_mod):
    """H=24, L=118800, d=128, M=128, N=1, 80% sparsity; the final query block has 16 rows."""
    w = W.HUNYUAN
    assert w.L % w.M == 16
    run_config(oracle_mod, w, n_random=72, closed_form_heads=(0, 13, 23))
