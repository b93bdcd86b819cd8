"""Host-side checks of the seeded input generators (no attention arithmetic involved)."""
import dataclasses

import numpy as np
import pytest

from paper_2509_16518_amd import workloads as W


def rows_of(indptr, indices):
    return [indices[indptr[i]:indptr[i + 1]] for i in range(indptr.size - 1)]


def test_normal_bf16_is_deterministic_and_standard():
    a = W.normal_bf16(5, 1, (1000, 64))
    b = W.normal_bf16(5, 1, (1000, 64))
    c = W.normal_bf16(5, 2, (1000, 64))
    assert (a == b).all() and (a != c).any()
    x = W.bf16_bits_to_f64(a)
    assert abs(x.mean()) < 0.02 and abs(x.std() - 1.0) < 0.02 and np.isfinite(x).all()
    # prefix property of a counter-based stream
    assert (W.normal_bf16(5, 1, (100,)) == a.reshape(-1)[:100]).all()


def test_bf16_round_trip_helpers():
    x = np.array([1.0, -2.5, 3.140625, 1e-3, 65280.0], dtype=np.float32)
    bits = W.f32_to_bf16_bits(x)
    back = W.bf16_bits_to_f64(bits)
    assert np.all(np.abs(back - x) <= np.abs(x) * 2.0 ** -8)
    assert (W.f32_to_bf16_bits(back.astype(np.float32)) == bits).all()
    # ties to even: 1 + 2^-8 sits between 1 and 1 + 2^-7
    assert W.bf16_bits_to_f64(W.f32_to_bf16_bits(np.array([1.0 + 2.0 ** -8], np.float32)))[0] == 1.0


def test_tiny_window_mask_shape_and_density():
    w = W.TINY
    indptr, indices = W.make_mask(w)
    assert indptr.shape == (w.items + 1,) and indptr[0] == 0 and indptr[-1] == indices.size
    dens = indices.size / (w.items * w.G)
    assert abs(dens - 0.30) < 0.01
    for i, r in enumerate(rows_of(indptr, indices)):
        assert r.size > 0 and (np.diff(r) > 0).all() and r[0] >= 0 and r[-1] < w.G
        # the window around the block's centre token is always present
        c = (i % w.QB) * w.M + w.M // 2
        ct, ch, cw = c // 256, (c // 16) % 16, c % 16
        for dt in (-1, 0, 1):
            for dh in (-3, 0, 3):
                for dw in (-3, 0, 3):
                    t, h, x = ct + dt, ch + dh, cw + dw
                    if 0 <= t < 4 and 0 <= h < 16 and 0 <= x < 16:
                        assert (t * 16 + h) * 16 + x in r
    again = W.make_mask(w)
    assert (again[0] == indptr).all() and (again[1] == indices).all()


@pytest.mark.parametrize("M,N", [(16, 1), (64, 8), (128, 32), (16, 64)])
def test_sweep_masks_valid(M, N):
    for kind in (W.MASK_WINDOW_FILL, W.MASK_RANDOM, W.MASK_ALL):
        w = W.sweep(M, N, kind)
        indptr, indices = W.make_mask(w)
        assert indptr.shape == (w.items + 1,)
        for r in rows_of(indptr, indices):
            assert (np.diff(r) > 0).all() and (r.size == 0 or (r[0] >= 0 and r[-1] < w.G))
        dens = indices.size / (w.items * w.G)
        if kind == W.MASK_ALL:
            assert dens == 1.0
        elif kind == W.MASK_RANDOM:
            assert abs(dens - 0.30) < 0.05
        else:
            assert dens >= 0.29          # window groups can push coarse masks above the target


def test_partial_blocks_and_groups():
    w = dataclasses.replace(W.TINY, L=1000, M=64, N=48, kind=W.MASK_RANDOM, grid=(1, 1, 1))
    indptr, indices = W.make_mask(w)
    assert w.QB == 16 and w.G == 21 and indptr.shape == (2 * 16 + 1,)
    assert indices.max() <= 20


def test_skew_len_generator_hits_its_bounds():
    w = dataclasses.replace(W.TINY, L=4096, M=128, N=32, kind=W.MASK_SKEW_LEN, skew=0.5, density=0.3, grid=(1, 1, 1))
    indptr, indices = W.make_mask(w)
    n = np.diff(indptr)
    lmax = 2 * 0.3 * w.G / (2 - 0.5)
    assert n.max() <= round(lmax) and n.min() >= round(0.5 * lmax) - 1
    assert abs(n.mean() / w.G - 0.3) < 0.03
    for r in rows_of(indptr, indices):
        assert (np.diff(r) > 0).all()


def test_skew_heads_varies_density_per_head():
    w = dataclasses.replace(W.WAN_14B_SKEW, H=6, L=4 * 12 * 16, grid=(4, 12, 16), window=(1, 2, 2))
    indptr, indices = W.make_mask(w)
    per_head = np.diff(indptr).reshape(6, -1).mean(axis=1) / w.G
    assert per_head.max() / per_head.min() > 1.3
    assert (per_head > 0.04).all() and (per_head < 0.99).all()


def test_flop_accounting():
    w = dataclasses.replace(W.TINY, L=1000, M=64, N=48, kind=W.MASK_ALL, grid=(1, 1, 1))
    indptr, indices = W.make_mask(w)
    assert (W.active_keys_per_item(w, indptr, indices) == 1000).all()
    assert W.useful_flop(w, indptr, indices) == W.dense_flop(w) == 4.0 * 64 * 1000 * 1000 * 2
