"""Pins for the fp64 oracle: each test fixes it to something other than itself.

The paper prints no worked numeric example for the kernel, so the pins are the ones the
mathematics gives: brute force over the full score matrix, a library attention routine,
closed forms and invariances.  Together they are chosen so that a dropped term, a wrong
sign or index, a transposed operand or a wrong group->key expansion fails at least one.
"""
import math

import numpy as np
import pytest
import torch

from paper_2509_16518_amd import workloads as W


def rand_bits(rng, shape, lo=-2.0, hi=2.0):
    return W.f32_to_bf16_bits(rng.uniform(lo, hi, size=shape).astype(np.float32))


def random_csr(rng, slices, L, M, N, density, allow_empty=False):
    QB, G = -(-L // M), -(-L // N)
    rows = []
    for _ in range(slices * QB):
        sel = np.flatnonzero(rng.random(G) < density).astype(np.int32)
        if sel.size == 0 and not allow_empty:
            sel = np.array([rng.integers(G)], dtype=np.int32)
        rows.append(sel)
    indptr = np.zeros(len(rows) + 1, dtype=np.int64)
    indptr[1:] = np.cumsum([r.size for r in rows])
    return indptr, (np.concatenate(rows) if rows else np.zeros(0, np.int32))


def key_level_bool_mask(L, M, N, indptr, indices, slices):
    """[slices, L, L] boolean: True where query row r may attend key k."""
    QB = -(-L // M)
    mask = np.zeros((slices, L, L), dtype=bool)
    for w in range(slices * QB):
        s, i = divmod(w, QB)
        for g in indices[indptr[w]:indptr[w + 1]]:
            mask[s, i * M:min((i + 1) * M, L), g * N:min((g + 1) * N, L)] = True
    return mask


def brute_force(qb, kb, vb, scale, mask):
    """Full L x L score matrix, elementwise -inf masking, row softmax, matmul (numpy, fp64)."""
    q, k, v = (W.bf16_bits_to_f64(x) for x in (qb, kb, vb))
    s = scale * np.einsum("sld,smd->slm", q, k)
    s = np.where(mask, s, -np.inf)
    m = s.max(axis=-1, keepdims=True)
    e = np.exp(s - m)
    z = e.sum(axis=-1, keepdims=True)
    return np.einsum("slm,smd->sld", e / z, v), (m + np.log(z))[..., 0]


def blocks_to_rows(out, lse, slices, L, M):
    """[items, M, d] / [items, M] -> [slices, L, d] / [slices, L] (drop rows past L)."""
    QB = -(-L // M)
    d = out.shape[-1]
    o = out.reshape(slices, QB * M, d)[:, :L]
    l = lse.reshape(slices, QB * M)[:, :L]
    return o, l


@pytest.mark.parametrize("L,M,N,d", [(32, 16, 1, 64), (30, 16, 4, 32), (29, 8, 3, 16), (17, 16, 17, 8)])
def test_brute_force_tiny(oracle_mod, L, M, N, d):
    rng = np.random.default_rng(7 + L + N)
    S = 2
    q, k, v = (rand_bits(rng, (S, L, d)) for _ in range(3))
    indptr, indices = random_csr(rng, S, L, M, N, 0.4)
    out, lse = oracle_mod.attention(q, k, v, M, N, 0.37, indptr, indices)
    o, l = blocks_to_rows(out, lse, S, L, M)
    ro, rl = brute_force(q, k, v, 0.37, key_level_bool_mask(L, M, N, indptr, indices, S))
    np.testing.assert_allclose(o, ro, rtol=0, atol=1e-12)
    np.testing.assert_allclose(l, rl, rtol=0, atol=1e-12)
    # rows past L stay NaN (never written)
    assert np.isnan(out.reshape(S, -1, d)[:, L:]).all()


def test_all_active_is_dense_sdpa(oracle_mod):
    """An all-active mask is textbook softmax attention: compare with torch's fp64 routine."""
    rng = np.random.default_rng(11)
    S, L, d, M, N = 3, 200, 64, 64, 8
    q, k, v = (rand_bits(rng, (S, L, d)) for _ in range(3))
    QB, G = -(-L // M), -(-L // N)
    indptr = np.arange(S * QB + 1, dtype=np.int64) * G
    indices = np.tile(np.arange(G, dtype=np.int32), S * QB)
    scale = 1 / math.sqrt(d)
    out, lse = oracle_mod.attention(q, k, v, M, N, scale, indptr, indices)
    o, l = blocks_to_rows(out, lse, S, L, M)
    tq, tk, tv = (torch.from_numpy(W.bf16_bits_to_f64(x)) for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=scale)
    np.testing.assert_allclose(o, ref.numpy(), rtol=0, atol=1e-12)
    ref_lse = torch.logsumexp(scale * tq @ tk.transpose(-1, -2), dim=-1)
    np.testing.assert_allclose(l, ref_lse.numpy(), rtol=0, atol=1e-12)


@pytest.mark.parametrize("N", [1, 4])
def test_masked_equals_sdpa_with_bool_mask(oracle_mod, N):
    """N = 1 is per-key -inf masking; N > 1 expands each group id to N consecutive keys."""
    rng = np.random.default_rng(13 + N)
    S, L, d, M = 2, 150, 32, 16
    q, k, v = (rand_bits(rng, (S, L, d)) for _ in range(3))
    indptr, indices = random_csr(rng, S, L, M, N, 0.3)
    out, lse = oracle_mod.attention(q, k, v, M, N, 0.25, indptr, indices)
    o, _ = blocks_to_rows(out, lse, S, L, M)
    mask = torch.from_numpy(key_level_bool_mask(L, M, N, indptr, indices, S))
    tq, tk, tv = (torch.from_numpy(W.bf16_bits_to_f64(x)) for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask, scale=0.25)
    np.testing.assert_allclose(o, ref.numpy(), rtol=0, atol=1e-12)


def test_group_mask_equals_expanded_key_mask(oracle_mod):
    """A group-level mask (N = 8) and its key-level expansion (N = 1) give the same result."""
    rng = np.random.default_rng(17)
    S, L, d, M, N = 2, 100, 16, 16, 8       # L % N != 0: the last group is short
    q, k, v = (rand_bits(rng, (S, L, d)) for _ in range(3))
    indptr, indices = random_csr(rng, S, L, M, N, 0.35)
    rows = [np.concatenate([np.arange(g * N, min((g + 1) * N, L)) for g in indices[indptr[w]:indptr[w + 1]]])
            for w in range(indptr.size - 1)]
    ip1 = np.zeros_like(indptr)
    ip1[1:] = np.cumsum([r.size for r in rows])
    a = oracle_mod.attention(q, k, v, M, N, 0.3, indptr, indices)
    b = oracle_mod.attention(q, k, v, M, 1, 0.3, ip1, np.concatenate(rows).astype(np.int32))
    np.testing.assert_array_equal(a[0], b[0])
    np.testing.assert_array_equal(a[1], b[1])


def test_single_active_key_returns_its_value_row(oracle_mod):
    rng = np.random.default_rng(19)
    S, L, d, M = 2, 64, 32, 16
    q, k, v = (rand_bits(rng, (S, L, d)) for _ in range(3))
    QB = L // M
    pick = rng.integers(0, L, size=S * QB).astype(np.int32)
    indptr = np.arange(S * QB + 1, dtype=np.int64)
    out, lse = oracle_mod.attention(q, k, v, M, 1, 0.5, indptr, pick)
    fq, fk, fv = (W.bf16_bits_to_f64(x) for x in (q, k, v))
    for w in range(S * QB):
        s, i = divmod(w, QB)
        np.testing.assert_array_equal(out[w], np.broadcast_to(fv[s, pick[w]], (M, d)))
        np.testing.assert_allclose(lse[w], 0.5 * fq[s, i * M:(i + 1) * M] @ fk[s, pick[w]], rtol=0, atol=1e-13)


def test_permutation_invariance(oracle_mod):
    rng = np.random.default_rng(23)
    S, L, d, M, N = 1, 96, 16, 32, 2
    q, k, v = (rand_bits(rng, (S, L, d)) for _ in range(3))
    indptr, indices = random_csr(rng, S, L, M, N, 0.5)
    shuffled = indices.copy()
    for w in range(indptr.size - 1):
        rng.shuffle(shuffled[indptr[w]:indptr[w + 1]])
    a = oracle_mod.attention(q, k, v, M, N, 0.2, indptr, indices)
    b = oracle_mod.attention(q, k, v, M, N, 0.2, indptr, shuffled)
    np.testing.assert_allclose(a[0], b[0], rtol=0, atol=1e-13)
    np.testing.assert_allclose(a[1], b[1], rtol=0, atol=1e-13)


def test_zero_query_closed_form(oracle_mod):
    """Q = 0: every weight is 1/|A|, so out = mean of the active V rows and lse = ln|A|."""
    rng = np.random.default_rng(29)
    S, L, d, M, N = 2, 120, 16, 16, 4
    q = np.zeros((S, L, d), dtype=np.uint16)
    k, v = (rand_bits(rng, (S, L, d)) for _ in range(2))
    indptr, indices = random_csr(rng, S, L, M, N, 0.3)
    out, lse = oracle_mod.attention(q, k, v, M, N, 0.7, indptr, indices)
    fv = W.bf16_bits_to_f64(v)
    QB = -(-L // M)
    for w in range(S * QB):
        s, i = divmod(w, QB)
        keys = np.concatenate([np.arange(g * N, min((g + 1) * N, L)) for g in indices[indptr[w]:indptr[w + 1]]])
        rows = min(M, L - i * M)
        np.testing.assert_allclose(out[w, :rows], np.broadcast_to(fv[s, keys].mean(0), (rows, d)), rtol=0, atol=1e-14)
        np.testing.assert_allclose(lse[w, :rows], math.log(keys.size), rtol=0, atol=1e-14)


def test_common_key_shift_moves_lse_only(oracle_mod):
    """Adding one vector c to every key shifts each row's scores by scale*<q,c>: out unchanged, lse shifted."""
    rng = np.random.default_rng(31)
    S, L, d, M = 1, 48, 8, 16
    ints = lambda lo, hi, shape: W.f32_to_bf16_bits(rng.integers(lo, hi, size=shape).astype(np.float32))
    q, k, v = ints(-3, 4, (S, L, d)), ints(-3, 4, (S, L, d)), ints(-8, 9, (S, L, d))
    c = rng.integers(-2, 3, size=d).astype(np.float64)
    k2 = W.f32_to_bf16_bits((W.bf16_bits_to_f64(k) + c).astype(np.float32))    # small integers: exact in bf16
    indptr, indices = random_csr(rng, S, L, M, 1, 0.5)
    a = oracle_mod.attention(q, k, v, M, 1, 0.125, indptr, indices)
    b = oracle_mod.attention(q, k2, v, M, 1, 0.125, indptr, indices)
    np.testing.assert_allclose(a[0], b[0], rtol=0, atol=1e-12)
    shift = 0.125 * W.bf16_bits_to_f64(q)[0] @ c
    np.testing.assert_allclose(b[1].reshape(-1)[:L] - a[1].reshape(-1)[:L], shift, rtol=0, atol=1e-12)


def test_scale_is_applied_to_scores_not_values(oracle_mod):
    """Two active keys: weights are the logistic function of scale*(s1 - s2)."""
    q = W.f32_to_bf16_bits(np.array([[[1.0, 2.0]] * 16], dtype=np.float32))           # [1,16,2]
    k = W.f32_to_bf16_bits(np.array([[[3.0, -1.0]] + [[0.5, 0.25]] * 15], dtype=np.float32))
    v = W.f32_to_bf16_bits(np.array([[[8.0, -4.0]] + [[2.0, 16.0]] * 15], dtype=np.float32))
    out, lse = oracle_mod.attention(q, k, v, 16, 1, 2.0, np.array([0, 2], np.int64), np.array([0, 5], np.int32))
    s1, s2 = 2.0 * (3.0 - 2.0), 2.0 * (0.5 + 0.5)
    w1 = 1.0 / (1.0 + math.exp(s2 - s1))
    np.testing.assert_allclose(out[0, 3], [w1 * 8 + (1 - w1) * 2, w1 * -4 + (1 - w1) * 16], rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse[0, 3], math.log(math.exp(s1) + math.exp(s2)), rtol=0, atol=1e-13)


def test_empty_list_gives_zero_and_minus_inf(oracle_mod):
    rng = np.random.default_rng(37)
    S, L, d, M = 1, 32, 8, 16
    q, k, v = (rand_bits(rng, (S, L, d)) for _ in range(3))
    indptr = np.array([0, 0, 3], dtype=np.int64)
    out, lse = oracle_mod.attention(q, k, v, M, 1, 1.0, indptr, np.array([1, 5, 9], np.int32))
    assert (out[0] == 0).all() and np.isneginf(lse[0]).all()
    assert np.isfinite(out[1]).all() and np.isfinite(lse[1]).all()


def test_rejects_out_of_range_group(oracle_mod):
    z = np.zeros((1, 16, 8), dtype=np.uint16)
    with pytest.raises(ValueError):
        oracle_mod.attention(z, z, z, 16, 1, 1.0, np.array([0, 1], np.int64), np.array([16], np.int32))


def test_sampled_items_match_full_run(oracle_mod):
    w = W.TINY
    q, k, v = W.make_qkv(w)
    indptr, indices = W.make_mask(w)
    full = oracle_mod.attention(q, k, v, w.M, w.N, w.scale, indptr, indices)
    pick = np.array([0, 63, 64, 127, 5], dtype=np.int64)
    part = oracle_mod.attention(q, k, v, w.M, w.N, w.scale, indptr, indices, items=pick)
    np.testing.assert_array_equal(full[0][pick], part[0])
    np.testing.assert_array_equal(full[1][pick], part[1])


def test_golden_regression_fixture(oracle_mod):
    """The stored values were written by tests/golden/make_golden.py, which calls only the oracle."""
    import os
    here = os.path.dirname(os.path.abspath(__file__))
    stored = np.loadtxt(os.path.join(here, "golden", "oracle_tiny_item5.txt"))
    w = W.TINY
    q, k, v = W.make_qkv(w)
    indptr, indices = W.make_mask(w)
    out, lse = oracle_mod.attention(q, k, v, w.M, w.N, w.scale, indptr, indices, items=np.array([5]))
    np.testing.assert_allclose(np.concatenate([out[0].reshape(-1), lse[0].reshape(-1)]), stored, rtol=1e-13, atol=1e-15)
