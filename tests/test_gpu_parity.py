"""Parity of the HIP path (through the C ABI) against the fp64 oracle, element by element.

Small cases run the oracle on every row; they span several LDS tiles, a ragged last tile, a
partial last query block and a short last key group.  Tolerances are the task's: out max-abs
<= 2e-2 and mean-abs <= 2e-3, lse within 1e-3 relative (see gpu_util).
"""
import dataclasses

import numpy as np
import pytest
import torch

from paper_2509_16518_amd import fgattn as F
from paper_2509_16518_amd import workloads as W
from gpu_util import Problem, check_against_oracle, compare, gather_items, out_to_f64, say, to_dev_bf16

pytestmark = pytest.mark.gpu


def small(M, N, d, L=1000, H=2, kind=W.MASK_RANDOM, density=0.3, seed=11, **kw):
    return dataclasses.replace(W.TINY, name="small-M%d-N%d-d%d-L%d" % (M, N, d, L), H=H, L=L, d=d, M=M, N=N, kind=kind,
                               density=density, seed=seed, grid=(1, 1, 1), **kw)


def test_tiny_config(oracle_mod):
    """Config 'Tiny': every row against the oracle."""
    prob = Problem(W.TINY)
    say("tiny: sparse forward")
    check_against_oracle(oracle_mod, prob, prob.run(), what="tiny")


@pytest.mark.parametrize("M", [16, 64, 128])
@pytest.mark.parametrize("N", [1, 8, 32, 64])
@pytest.mark.parametrize("kind", [W.MASK_WINDOW_FILL, W.MASK_RANDOM])
def test_tile_granularity_sweep(oracle_mod, M, N, kind):
    w = W.sweep(M, N, kind)
    say("sweep %s" % w.name)
    prob = Problem(w)
    check_against_oracle(oracle_mod, prob, prob.run(), what=w.name)


@pytest.mark.parametrize("M,d", [(16, 64), (32, 64), (64, 64), (128, 64), (16, 128), (32, 128), (64, 128), (128, 128)])
def test_all_active_equals_dense_kernel_and_oracle(oracle_mod, M, d):
    """0% sparsity: the sparse entry point with an all-active mask, the dense entry point and the oracle agree."""
    w = small(M, 1, d, L=777, kind=W.MASK_ALL)
    say("all-active %s" % w.name)
    prob = Problem(w)
    sparse = prob.run()
    check_against_oracle(oracle_mod, prob, sparse, what=w.name + " sparse-entry")
    dense = prob.run(dense=True)
    check_against_oracle(oracle_mod, prob, dense, what=w.name + " dense-entry")
    # same keys in the same order through the same arithmetic: bit-identical
    assert np.array_equal(sparse[0], dense[0]) and np.array_equal(sparse[1], dense[1])


@pytest.mark.parametrize("M,N,d,L", [(64, 48, 128, 1000), (16, 7, 64, 333), (128, 3, 128, 517), (32, 5, 64, 2049),
                                      (64, 1, 128, 65), (128, 1, 64, 1), (16, 1, 128, 15), (32, 1000, 64, 1000)])
def test_ragged_shapes(oracle_mod, M, N, d, L):
    """Partial last query block, short last key group (L % N != 0), N not a power of two, L < M, one group."""
    w = small(M, N, d, L=L, density=0.45)
    say("ragged %s" % w.name)
    prob = Problem(w)
    rc = F.fgattn_validate_mask(prob.d_indptr, prob.d_indices, prob.params(), prob.workspace(prob.params()))
    assert rc == 0
    check_against_oracle(oracle_mod, prob, prob.run(), what=w.name)


def test_short_last_group_in_the_middle_of_an_unsorted_list(oracle_mod):
    w = small(64, 48, 128, L=1000, density=0.6, seed=21)
    prob0 = Problem(w)
    rng = np.random.default_rng(5)
    ind = prob0.indices.copy()
    for i in range(w.items):
        rng.shuffle(ind[prob0.indptr[i]:prob0.indptr[i + 1]])
    prob = Problem(w, prob0.q_bits, prob0.k_bits, prob0.v_bits, mask=(prob0.indptr, ind))
    got = prob.run()
    check_against_oracle(oracle_mod, prob, got, what="unsorted short group")
    # permutation invariance against the sorted run, within tolerance (summation order differs)
    ref = prob0.run()
    assert np.nanmax(np.abs(got[0] - ref[0])) <= 2e-2 and np.nanmax(np.abs(got[1] - ref[1])) <= 1e-3


def test_empty_and_single_key_lists(oracle_mod):
    """An empty list gives out = 0 and lse = -inf (never NaN); one active key returns that V row exactly."""
    w = small(64, 1, 128, L=500, seed=31)
    q, k, v = W.make_qkv(w)
    rng = np.random.default_rng(3)
    rows = []
    for i in range(w.items):
        kind = i % 3
        rows.append(np.zeros(0, np.int32) if kind == 0 else
                    rng.integers(0, w.G, size=1).astype(np.int32) if kind == 1 else
                    np.sort(rng.choice(w.G, size=70, replace=False)).astype(np.int32))
    indptr = np.zeros(w.items + 1, np.int64)
    indptr[1:] = np.cumsum([r.size for r in rows])
    prob = Problem(w, q, k, v, mask=(indptr, np.concatenate(rows)))
    got = prob.run()
    check_against_oracle(oracle_mod, prob, got, what="empty/single")
    bo, bl = gather_items(w, got[0], got[1], np.arange(w.items))
    fv = W.bf16_bits_to_f64(v).reshape(-1, w.L, w.d)
    for i in range(w.items):
        nrow = min(w.M, w.L - (i % w.QB) * w.M)
        if i % 3 == 0:
            assert (bo[i, :nrow] == 0).all() and np.isneginf(bl[i, :nrow]).all()
        elif i % 3 == 1:
            assert (bo[i, :nrow] == fv[i // w.QB, rows[i][0]]).all()     # bit-exact V row


def test_all_lists_empty():
    w = small(16, 1, 64, L=100, seed=33)
    q, k, v = W.make_qkv(w)
    prob = Problem(w, q, k, v, mask=(np.zeros(w.items + 1, np.int64), np.zeros(0, np.int32)))
    out, lse = prob.run()
    assert (out == 0).all() and np.isneginf(lse).all()


@pytest.mark.parametrize("M,d", [(64, 128), (128, 64), (16, 64)])
def test_spike_at_tile_boundaries(oracle_mod, M, d):
    """One key dominates the softmax; it is placed at list positions around the LDS tile edges and at the
    ragged tail, for list lengths = 0, 1, -1 (mod tile).  out must be its V row and lse its score."""
    NT = {16: 128, 32: 128, 64: 64, 128: 64}[M]
    w0 = small(M, 1, d, L=2048, H=1, seed=41)
    q, k, v = W.make_qkv(w0)
    fq, fk = W.bf16_bits_to_f64(q)[0, 0], W.bf16_bits_to_f64(k)[0, 0]
    rng = np.random.default_rng(9)
    rows, spikes = [], []
    spike_key = 2047
    lengths = [3 * NT, 3 * NT + 1, 3 * NT - 1, NT, NT + 1, 1, 2, NT - 1]
    for i in range(w0.QB):
        n = lengths[i % len(lengths)]
        pos = [0, NT - 1, NT, n - 1, n // 2][(i // len(lengths)) % 5] % n
        others = rng.choice(2047, size=n - 1, replace=False).astype(np.int32)
        lst = np.insert(others, pos, spike_key).astype(np.int32)
        rows.append(lst)
        spikes.append(pos)
    # spike key: same direction as every query of... each block has different queries, so use a constant
    # query direction instead: all queries = 4 * e_0 + noise-free pattern; spike key = 8 * e_0.
    qc = np.zeros_like(fq)
    qc[:, 0] = 4.0
    qc[:, 1:] = fq[:, 1:] * 0.25
    kc = fk * 0.25
    kc[spike_key] = 0
    kc[spike_key, 0] = 64.0
    qb = W.f32_to_bf16_bits(qc.astype(np.float32)).reshape(q.shape)
    kb = W.f32_to_bf16_bits(kc.astype(np.float32)).reshape(k.shape)
    indptr = np.zeros(w0.items + 1, np.int64)
    indptr[1:] = np.cumsum([r.size for r in rows])
    prob = Problem(w0, qb, kb, v, mask=(indptr, np.concatenate(rows)))
    got = prob.run(scale=1.0)
    check_against_oracle(oracle_mod, prob, got, what="spike M%d d%d" % (M, d), scale=1.0)
    fv = W.bf16_bits_to_f64(v)[0, 0]
    assert (got[0][0, 0] == fv[spike_key]).all()            # every row returns the spike's V row exactly
    np.testing.assert_allclose(got[1][0, 0], 256.0, rtol=0, atol=1e-3)


@pytest.mark.parametrize("ascending", [True, False])
def test_running_max_arrives_last_or_first(oracle_mod, ascending):
    """Planted scores grow (or shrink) along the list, so the online-softmax rescale runs on every tile."""
    w = small(64, 1, 128, L=1536, H=1, seed=51, kind=W.MASK_ALL)
    q, k, v = W.make_qkv(w)
    fk = W.bf16_bits_to_f64(k)[0, 0] * 0.125
    ramp = np.linspace(0.0, 12.0, w.L) if ascending else np.linspace(12.0, 0.0, w.L)
    fk[:, 0] = ramp
    fq = W.bf16_bits_to_f64(q)[0, 0] * 0.125
    fq[:, 0] = 2.0
    prob = Problem(w, W.f32_to_bf16_bits(fq.astype(np.float32)).reshape(q.shape),
                   W.f32_to_bf16_bits(fk.astype(np.float32)).reshape(k.shape), v)
    check_against_oracle(oracle_mod, prob, prob.run(scale=1.0), what="ramp asc=%s" % ascending, scale=1.0)


@pytest.mark.parametrize("scale", [-0.09, 0.0, 0.5])
def test_scale_sign_and_zero(oracle_mod, scale):
    w = small(64, 4, 128, L=600, seed=61)
    prob = Problem(w)
    check_against_oracle(oracle_mod, prob, prob.run(scale=scale), what="scale %g" % scale, scale=scale)


def test_group_mask_equals_expanded_key_mask(oracle_mod):
    """N = 8 group mask vs its N = 1 key-level expansion: same keys, same order -> bit-identical output."""
    w8 = small(64, 8, 128, L=1000, seed=71)
    p8 = Problem(w8)
    rows = [np.concatenate([np.arange(g * 8, min(g * 8 + 8, w8.L)) for g in p8.indices[p8.indptr[i]:p8.indptr[i + 1]]])
            .astype(np.int32) if p8.indptr[i + 1] > p8.indptr[i] else np.zeros(0, np.int32) for i in range(w8.items)]
    ip1 = np.zeros(w8.items + 1, np.int64)
    ip1[1:] = np.cumsum([r.size for r in rows])
    w1 = dataclasses.replace(w8, N=1)
    p1 = Problem(w1, p8.q_bits, p8.k_bits, p8.v_bits, mask=(ip1, np.concatenate(rows)))
    a, b = p8.run(), p1.run()
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    check_against_oracle(oracle_mod, p8, a, what="N=8")


def test_batch_and_strided_layout(oracle_mod):
    """B = 2 and [B, L, H, d] memory layout (heads interleaved) through the stride arguments."""
    w = dataclasses.replace(small(64, 2, 128, L=520, H=3, seed=81), B=2)
    prob = Problem(w)
    ref = prob.run()
    check_against_oracle(oracle_mod, prob, ref, what="B=2 contiguous")
    tr = lambda t: t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)      # same values, [B,L,H,d] storage
    q2, k2, v2 = tr(prob.q), tr(prob.k), tr(prob.v)
    out2 = torch.empty_like(q2.permute(0, 2, 1, 3).contiguous()).permute(0, 2, 1, 3)
    assert q2.stride(1) == w.d and q2.stride(2) == w.H * w.d
    p = prob.params(q=q2, k=k2, v=v2, out=out2)
    lse2 = torch.empty_like(prob.lse)
    F.fgattn_forward(q2, k2, v2, prob.d_indptr, prob.d_indices, p, out2, lse2, prob.workspace(p))
    torch.cuda.synchronize()
    assert np.array_equal(out_to_f64(out2.contiguous()), ref[0])
    assert np.array_equal(lse2.double().cpu().numpy(), ref[1])


@pytest.mark.parametrize("M,N", [(64, 1), (128, 8)])
def test_gather_offsets_up_to_the_4_gib_limit(oracle_mod, M, N):
    """K and V rows one MiB apart: the byte offset of the last row is just below 2^32, the largest the 32-bit
    gather offsets take (row stride below 16 MiB, last row + 4 KiB inside 4 GiB), and far above 2^31."""
    L, d, stride_l = 4096, 128, 1 << 19                      # elements: 1 MiB per row
    assert (L - 1) * stride_l * 2 + 2 * d + 4096 <= 0xFFFFFFFF < L * stride_l * 2 + 2 * d + 4096
    w = small(M, N, d, L=L, H=1, seed=87)
    prob = Problem(w)

    def spread(t):   # same values, rows one MiB apart (only the rows themselves are ever written or read)
        big = torch.empty(L * stride_l, dtype=torch.bfloat16, device="cuda")
        view = big.as_strided((1, 1, L, d), (L * stride_l, L * stride_l, stride_l, 1))
        view.copy_(t)
        return view

    k2, v2 = spread(prob.k), spread(prob.v)
    p = prob.params(k=k2, v=v2)
    assert p.k_stride_l == stride_l and p.v_stride_l == stride_l
    prob.out.view(torch.int16).fill_(0x7FC0)
    prob.lse.fill_(float("nan"))
    say("offsets up to 4 GiB M=%d N=%d" % (M, N))
    F.fgattn_forward(prob.q, k2, v2, prob.d_indptr, prob.d_indices, p, prob.out, prob.lse, prob.workspace(p))
    torch.cuda.synchronize()
    got = (out_to_f64(prob.out), prob.lse.double().cpu().numpy())
    check_against_oracle(oracle_mod, prob, got, what="rows 1 MiB apart")
    # and bit for bit what the contiguous layout gives
    ref = prob.run()
    assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])
    del k2, v2
    torch.cuda.empty_cache()


def test_maximum_sequence_length(oracle_mod):
    """L = 2^24, the longest sequence the boundary takes (key rows are multiplied as 24-bit numbers): d = 64 keeps a
    K/V slice at 2 GiB.  131072 query blocks of one head (the ordering pre-pass sorts them by buckets), 48 keys each,
    with the first and the last key of the sequence in many lists; sampled items against the oracle."""
    L, M, d, per = 1 << 24, 128, 64, 48
    w = dataclasses.replace(W.TINY, name="max-L", H=1, L=L, d=d, M=M, N=1, grid=(1, 1, 1), seed=97)
    say("L = 2^24: generating")
    q, k, v = W.make_qkv(w)
    rng = np.random.default_rng(5)
    items = w.items
    keys = rng.integers(1, L - 1, size=(items, per), dtype=np.int64)
    keys[::3, 0] = 0          # the first key ...
    keys[1::3, 0] = L - 1     # ... and the last one
    keys.sort(axis=1)
    # drop the (rare) duplicates inside a list: lists of slightly different lengths
    lists = [np.unique(row) for row in keys[:4096]]   # (the vectorised construction below is checked against these)
    keep = np.ones_like(keys, dtype=bool)
    keep[:, 1:] = keys[:, 1:] != keys[:, :-1]
    indptr = np.concatenate([[0], np.cumsum(keep.sum(1))]).astype(np.int64)
    indices = keys[keep].astype(np.int32)
    assert all(np.array_equal(indices[indptr[i]:indptr[i + 1]], lists[i]) for i in range(0, 4096, 97))
    prob = Problem(w, q, k, v, mask=(indptr, indices))
    p = prob.params()
    assert F.fgattn_validate_mask(prob.d_indptr, prob.d_indices, p, prob.workspace(p)) == 0
    say("L = 2^24: forward")
    got = prob.run()
    picks = np.array(sorted({0, 1, 2, items - 3, items - 2, items - 1} | set(rng.integers(0, items, size=26).tolist())), dtype=np.int64)
    check_against_oracle(oracle_mod, prob, got, items=picks, what="L = 2^24")
    # every row's lse is finite (no list is empty) and no row was left unwritten
    assert np.isfinite(got[1]).all()
    del prob
    torch.cuda.empty_cache()


def test_zero_query_closed_form_is_exact():
    """Q = 0: all weights are 1/|A| exactly, so out = bf16(mean of active V rows) and lse = ln|A|."""
    w = small(64, 1, 128, L=3000, H=2, seed=91, density=0.4)
    q, k, v = W.make_qkv(w)
    # V rows = small integers: fp32 accumulation is exact
    vi = (np.arange(w.L)[:, None] * 7 + np.arange(w.d)[None, :] * 3) % 17 - 8
    vb = np.broadcast_to(W.f32_to_bf16_bits(vi.astype(np.float32)), v.shape[:2] + vi.shape).copy()
    prob = Problem(w, np.zeros_like(q), k, vb)
    out, lse = prob.run()
    for i in range(w.items):
        s, b = divmod(i, w.QB)
        keys = prob.indices[prob.indptr[i]:prob.indptr[i + 1]]
        r0, r1 = b * w.M, min((b + 1) * w.M, w.L)
        mean = vi[keys].sum(0) / keys.size
        np.testing.assert_allclose(lse[0, s, r0:r1], np.log(keys.size), rtol=0, atol=2e-6 * np.log(keys.size) + 1e-6)
        assert np.all(np.abs(out[0, s, r0:r1] - mean) <= np.abs(mean) * 2.0 ** -8 + 1e-30)


def _random_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for c in range(n):
        M = int(rng.choice([16, 32, 64, 128]))
        d = int(rng.choice([64, 128]))
        N = int(rng.choice([1, 1, 2, 4, 8, 12, 16, 32, 33, 64, 100, 128]))
        L = int(rng.integers(1, 1800))
        H = int(rng.integers(1, 4))
        kind = [W.MASK_RANDOM, W.MASK_SKEW_LEN][int(rng.integers(0, 2))]
        density = float(rng.choice([0.05, 0.3, 0.6, 1.0]))
        cases.append((M, N, d, L, H, kind, density, 9000 + c))
    return cases


@pytest.mark.parametrize("M,N,d,L,H,kind,density,seed", _random_cases(24, 20250927))
def test_seeded_random_shapes(oracle_mod, M, N, d, L, H, kind, density, seed):
    """Shapes nobody picked by hand: tile size, group size (also not a power of two, larger than L), length, head
    count, list-length skew and density drawn from a fixed seed; every row against the oracle."""
    w = small(M, N, d, L=L, H=H, kind=kind, density=density, seed=seed, skew=0.8)
    say("random shape %s H=%d kind=%d density=%.2f" % (w.name, H, kind, density))
    prob = Problem(w)
    p = prob.params()
    assert F.fgattn_validate_mask(prob.d_indptr, prob.d_indices, p, prob.workspace(p)) == 0
    check_against_oracle(oracle_mod, prob, prob.run(), what=w.name)


def _wide_random_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for c in range(n):
        M = int(rng.choice([16, 32, 64, 128]))
        d = int(rng.choice([64, 128]))
        N = int(rng.choice([1, 1, 1, 2, 3, 4, 7, 8, 16, 31, 32, 64, 128, 200]))
        L = int(rng.integers(1, 5000))
        H = int(rng.integers(1, 10))
        B = int(rng.choice([1, 1, 2]))
        kind = [W.MASK_RANDOM, W.MASK_SKEW_LEN, W.MASK_WINDOW_FILL][int(rng.integers(0, 3))]
        density = float(rng.choice([0.02, 0.1, 0.3, 0.7, 1.0]))
        flags = int(rng.choice([0, 0, F.FLAG_STATIC_ASSIGN, F.FLAG_FIFO_QUEUE]))
        skew = float(rng.choice([0.0, 0.5, 1.0]))
        span = int(rng.integers(1, 40))
        cases.append((M, N, d, L, H, B, kind, density, flags, skew, span, 12000 + c))
    return cases


@pytest.mark.parametrize("M,N,d,L,H,B,kind,density,flags,skew,span,seed", _wide_random_cases(64, 20251128))
def test_seeded_random_shapes_wide(oracle_mod, M, N, d, L, H, B, kind, density, flags, skew, span, seed):
    """A wider draw than test_seeded_random_shapes: up to nine heads (more and fewer than the eight queues), B = 2,
    the three mask generators, densities from 2% to all keys, the three scheduling modes; every row against the oracle."""
    w = dataclasses.replace(small(M, N, d, L=L, H=H, kind=kind, density=density, seed=seed, skew=skew), B=B)
    if kind == W.MASK_WINDOW_FILL:
        w = dataclasses.replace(w, grid=(1, 1, L), window=(0, 0, span))
    say("wide random shape %s H=%d B=%d kind=%d density=%.2f flags=%d" % (w.name, H, B, kind, density, flags))
    prob = Problem(w)
    check_against_oracle(oracle_mod, prob, prob.run(flags=flags), what=w.name)
