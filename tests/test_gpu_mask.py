"""GPU parity of the top-p mask (paper Sec. 4.3) against the oracle, through the C ABI.

What is unique is compared exactly: the bf16 block means (bit for bit), and the kept set of every
query block whose cumulative probability clears p by more than rounding.  Where the oracle's
fp64 cumulative sum passes p within EPS of a boundary, the fp32/fixed-point kernel may keep one
key block more or fewer: there the kept set must still be a top set of the oracle's ranking (up to
EPS in probability) whose mass reaches p - EPS and would not reach p + EPS without its last member.
EPS = 1e-5 covers the fp32 accumulation of 128 exact bf16 products (relative 1e-6 on a score of
order 1, hence on a weight), the 1-ulp exp2 and the 2^-40 fixed point.
"""
import math

import numpy as np
import pytest
import torch

from paper_2509_16518_amd import fgattn as F
from paper_2509_16518_amd import workloads as W
from gpu_util import Problem, check_against_oracle, say, to_dev_bf16

pytestmark = pytest.mark.gpu
EPS = 1e-5
# Query blocks per test case (keyed by the label and p) whose kept set differed from the oracle's inside the
# rounding allowance above, as observed on the GPU.  Every case not listed has none and must stay at none: the
# allowance exists for cumulative sums that pass p within EPS, and is not a blanket budget.
OBSERVED_ROUNDING_ESCAPES = {
    # query block 1986 of the sampled ones: key blocks 42188 and 116081 straddle the cut with scores that are equal
    # in fp32 (the kernel's ranking precision: it keeps the lower id) and differ in the eighth digit in the oracle's
    # fp64; the kept sets differ by that one swap
    "hunyuan p=0.9": 1,
}


def gpu_mask(w, q_bits, k_bits, top_p, scale=None, want_pooled=False, flags=0):
    """Runs select + emit; returns (indptr, indices) as numpy (and the Q block means if asked)."""
    q, k = to_dev_bf16(q_bits), to_dev_bf16(k_bits)
    p = F.make_params(q, k, k, q, w.M, w.N, w.scale if scale is None else scale, flags)
    nbytes = F.fgattn_mask_workspace_bytes(p)
    assert nbytes > 0
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    rows = w.B * w.H * w.QB
    indptr = torch.full((rows + 1,), -1, dtype=torch.int64, device="cuda")
    F.fgattn_mask_select(q, k, p, top_p, indptr, ws)
    nnz = int(indptr[-1].item())
    assert nnz >= rows, "every query block keeps at least one key block"
    indices = torch.full((nnz + 8,), -7, dtype=torch.int32, device="cuda")   # 8 guard entries behind the capacity
    F.fgattn_mask_emit(p, indptr, indices[:nnz], ws)
    torch.cuda.synchronize()
    assert (indices[nnz:] == -7).all(), "emit wrote past the capacity"
    res = (indptr.cpu().numpy(), indices[:nnz].cpu().numpy())
    if want_pooled:
        pooled = ws[:rows * w.d * 2].view(torch.int16).cpu().numpy().view(np.uint16).reshape(w.B * w.H, w.QB, w.d)
        return res + (pooled,)
    return res


def check_rows(oracle, w, q_bits, k_bits, top_p, indptr, indices, rows, scale=None, what=""):
    """Compares the kept sets of the given query blocks with the oracle; returns the number that differed (validly)."""
    assert indptr[0] == 0 and np.all(np.diff(indptr) >= 1)
    # (the C ABI takes top_p and scale as floats: the oracle gets the same numbers, not the doubles they were rounded from)
    ref = oracle.topp_rows(q_bits, k_bits, w.M, w.N, float(np.float32(w.scale if scale is None else scale)),
                           float(np.float32(top_p)), rows=rows)
    inexact = 0
    for row, (kept, order, cum) in zip(rows, ref):
        got = indices[indptr[row]:indptr[row + 1]]
        assert np.all(np.diff(got) > 0) and got[0] >= 0 and got[-1] < w.G, "%s row %d: ids not ascending / in range" % (what, row)
        want = np.sort(order[:kept])
        if got.size == want.size and np.array_equal(got, want):
            continue
        inexact += 1
        prob = np.empty(w.G)
        prob[order] = np.diff(np.concatenate([[0.0], cum]))
        inside = np.zeros(w.G, dtype=bool)
        inside[got] = True
        lo_in, hi_out = prob[inside].min(), (prob[~inside].max() if (~inside).any() else 0.0)
        mass = prob[inside].sum()
        ok = lo_in >= hi_out - EPS and mass >= top_p - EPS and mass - lo_in < top_p + EPS
        assert ok, "%s row %d: kept %d (oracle %d), mass %.9f, least kept %.3e, best dropped %.3e" % (
            what, row, got.size, kept, mass, lo_in, hi_out)
    say("    %s: %d rows checked, %d differ within rounding of p" % (what, len(rows), inexact))
    key = "%s p=%g" % (what, top_p)
    assert inexact == OBSERVED_ROUNDING_ESCAPES.get(key, 0), "%s: %d query blocks used the rounding allowance" % (key, inexact)
    return inexact


@pytest.mark.parametrize("M,N,d,L,grid", [(16, 1, 64, 1024, (4, 16, 16)), (64, 8, 128, 1024, (4, 16, 16)),
                                          (128, 32, 128, 1024, (4, 16, 16)), (32, 1, 128, 1000, (10, 10, 10)),
                                          (64, 3, 64, 1000, (10, 10, 10)), (16, 1, 64, 3000, (3, 25, 40))])
@pytest.mark.parametrize("top_p", [0.5, 0.9])
@pytest.mark.parametrize("flags", [0, F.FLAG_MASK_ROWS_IN_HBM, F.FLAG_MASK_ONE_TILE_CHUNKS,
                                   F.FLAG_MASK_ROWS_IN_HBM | F.FLAG_MASK_ONE_TILE_CHUNKS],
                         ids=["lds-rows", "hbm-rows", "lds-rows-chunked", "hbm-rows-chunked"])
def test_mask_matches_oracle_small(oracle_mod, M, N, d, L, grid, top_p, flags):
    w = W.Workload("mask-M%d-N%d-d%d-L%d" % (M, N, d, L), H=2, L=L, d=d, M=M, N=N, grid=grid, seed=4000 + M + N)
    q, k = W.make_qk_local(w, gain=1.5 if d == 64 else 1.2)
    say("mask %s p=%.2f" % (w.name, top_p))
    indptr, indices, pooled = gpu_mask(w, q, k, top_p, want_pooled=True, flags=flags)
    assert np.array_equal(pooled, oracle_mod.pool(q, M)), "query block means differ from the oracle's bits"
    rows = list(range(w.items))
    bad = check_rows(oracle_mod, w, q, k, top_p, indptr, indices, rows, what=w.name)
    density = indices.size / float(w.items * w.G)
    say("    density %.3f" % density)


def test_mask_unstructured_inputs(oracle_mod):
    # plain N(0,1) Q, K: nearly flat probabilities, most key blocks are kept and many masses sit close together
    w = W.Workload("mask-flat", H=2, L=2048, d=128, M=64, N=1, seed=4100)
    q, k, _ = W.make_qkv(w)
    say("mask flat")
    indptr, indices = gpu_mask(w, q, k, 0.9)
    check_rows(oracle_mod, w, q, k, 0.9, indptr, indices, list(range(w.items)), what=w.name)


@pytest.mark.parametrize("L,N,top_p,kept,flags", [(1024, 8, 0.75, 96, 0), (8192, 1, 0.75, 6144, 0), (8192, 1, 0.5, 4096, 0),
                                                  (1024, 8, 0.75, 96, 8), (8192, 1, 0.5, 4096, 8),
                                                  (8192, 1, 0.5, 4096, 16), (40000, 1, 0.625, 25000, 16),
                                                  (40000, 1, 0.625, 25000, 0), (32768, 1, 0.5, 16384, 0),
                                                  (32767, 1, 0.5, 16384, 0), (32769, 1, 0.5, 16385, 0)])
def test_uniform_scores_closed_form(L, N, top_p, kept, flags):
    # Q = 0: all key blocks weigh the same, the mask is the ceil(p*G) lowest ids.  G = 128 goes through the
    # sorted-bin path, G = 8192 and 40000 through the run-of-equal-scores path (more members than fit the sort);
    # 40000 key blocks are more than a row kept in LDS holds, so that case selects from device memory by itself.
    # (32768 key blocks fill the LDS row exactly; one more takes the other path)
    w = W.Workload("mask-uniform", H=1, L=L, d=64, M=64 if L < 30000 else 128, N=N, seed=4200)
    _, k, _ = W.make_qkv(w)
    q = np.zeros_like(k)
    say("mask uniform L=%d N=%d p=%.2f" % (L, N, top_p))
    indptr, indices = gpu_mask(w, q, k, top_p, flags=flags)
    assert np.array_equal(np.diff(indptr), np.full(w.items, kept))
    for r in range(w.items):
        assert np.array_equal(indices[indptr[r]:indptr[r + 1]], np.arange(kept))


@pytest.mark.parametrize("L,flags", [(8192, 0), (8192, F.FLAG_MASK_ROWS_IN_HBM), (40000, 0), (40000, F.FLAG_MASK_ONE_TILE_CHUNKS)])
def test_clustered_scores_take_the_narrowing_rounds(oracle_mod, L, flags):
    # Ten key blocks score about ln(0.15 L) (together some 60-80% of the mass), all others within +-0.01 of zero: the
    # histogram over the score range puts the
    # whole crowd into one bin, which is also where the mass crosses p -- far more members than the ranking holds
    # (512 in the kernel that keeps the bins in LDS, which then hands the row over; 2048 in the general kernel), so
    # the bin is narrowed by re-histogramming its range of score bits and all bits are rewritten from the cut.
    w = W.Workload("mask-crowd-L%d" % L, H=1, L=L, d=128, M=128, N=1, seed=4400)
    rng = np.random.default_rng(L)
    kf = (1e-3 * rng.standard_normal((1, 1, L, w.d))).astype(np.float32)
    loud = rng.choice(L, size=10, replace=False)
    kf[0, 0, loud] = np.log(0.15 * L) / 64.0
    qf = np.empty((1, 1, L, w.d), dtype=np.float32)
    qf[0, 0] = (0.5 + 0.0002 * (np.arange(L) // w.M))[:, None]
    q, k = W.f32_to_bf16_bits(qf), W.f32_to_bf16_bits(kf)
    say("mask crowd L=%d flags=%d" % (L, flags))
    indptr, indices = gpu_mask(w, q, k, 0.9, scale=1.0, flags=flags)
    nnz = np.diff(indptr)
    assert nnz.min() > 2048 and nnz.max() < L - 2048, "the cut is meant to fall inside the crowd"
    for r in range(w.items):
        assert np.isin(loud, indices[indptr[r]:indptr[r + 1]]).all()
    rows = list(range(0, w.items, max(1, w.items // 12))) + [w.items - 1]
    check_rows(oracle_mod, w, q, k, 0.9, indptr, indices, rows, scale=1.0, what=w.name)


def test_dominant_key_block_and_p_one(oracle_mod):
    w = W.Workload("mask-spike", H=1, L=512, d=64, M=32, N=4, seed=4300)
    rng = np.random.default_rng(3)
    q = W.f32_to_bf16_bits(np.ones((1, 1, w.L, w.d), dtype=np.float32))
    kf = rng.uniform(-0.1, 0.1, size=(1, 1, w.L, w.d)).astype(np.float32)
    kf[0, 0, 5 * w.N:6 * w.N] = 4.0
    k = W.f32_to_bf16_bits(kf)
    say("mask spike")
    indptr, indices = gpu_mask(w, q, k, 0.9, scale=1.0)
    assert np.array_equal(np.diff(indptr), np.ones(w.items)) and np.all(indices == 5)
    # top_p = 1: everything that has any weight at 2^-40 resolution -- here every key block but nothing twice
    indptr, indices = gpu_mask(w, q, k, 1.0, scale=0.05)
    assert np.all(np.diff(indptr) <= w.G) and np.all(np.diff(indptr) >= 1)
    check_rows(oracle_mod, w, q, k, 1.0, indptr, indices, list(range(w.items)), scale=0.05, what="p=1")


def test_mask_rows_longer_than_lds(oracle_mod):
    # 33000 key blocks: above the 32768 that the LDS-row selection holds; sampled query blocks against the oracle
    w = W.Workload("mask-long-rows", H=1, L=33000, d=64, M=128, N=1, grid=(10, 55, 60), seed=4500)
    q, k = W.make_qk_local(w, gain=1.5)
    say("mask %s" % w.name)
    indptr, indices = gpu_mask(w, q, k, 0.9)
    rows = list(range(0, w.items, 13)) + [w.items - 1]
    bad = check_rows(oracle_mod, w, q, k, 0.9, indptr, indices, rows, what=w.name)
    say("    density %.3f" % (indices.size / float(w.items * w.G)))


@pytest.mark.parametrize("N", [1, 4])
def test_mask_batch_and_strided_layout(oracle_mod, N):
    # B = 2 with [B, L, H, d] storage (heads interleaved) through the stride arguments; last query block is short
    import dataclasses
    w = dataclasses.replace(W.Workload("mask-batch-N%d" % N, H=3, L=520, d=128, M=64, N=N, grid=(5, 8, 13), seed=4600 + N), B=2)
    q, k = W.make_qk_local(w, gain=1.2)
    say("mask %s, strided" % w.name)
    tr = lambda t: t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)      # same values, [B,L,H,d] storage
    dq, dk = tr(to_dev_bf16(q)), tr(to_dev_bf16(k))
    assert dq.stride(1) == w.d and dq.stride(2) == w.H * w.d
    p = F.make_params(dq, dk, dk, dq, w.M, w.N, w.scale)
    ws = torch.empty(F.fgattn_mask_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    rows = w.B * w.H * w.QB
    indptr = torch.full((rows + 1,), -1, dtype=torch.int64, device="cuda")
    F.fgattn_mask_select(dq, dk, p, 0.8, indptr, ws)
    nnz = int(indptr[-1].item())
    indices = torch.full((nnz,), -7, dtype=torch.int32, device="cuda")
    F.fgattn_mask_emit(p, indptr, indices, ws)
    torch.cuda.synchronize()
    pooled = ws[:rows * w.d * 2].view(torch.int16).cpu().numpy().view(np.uint16).reshape(w.B * w.H, w.QB, w.d)
    assert np.array_equal(pooled, oracle_mod.pool(q, w.M)), "query block means differ from the oracle's bits"
    bad = check_rows(oracle_mod, w, q, k, 0.8, indptr.cpu().numpy(), indices.cpu().numpy(), list(range(rows)), what=w.name)


def test_mask_feeds_forward(oracle_mod):
    # the loop closed on the device: Q, K -> mask -> sparse attention, checked against the oracle run on that mask
    w = W.Workload("mask-then-attend", H=2, L=1024, d=128, M=64, N=8, grid=(4, 16, 16), seed=4400)
    q, k = W.make_qk_local(w, gain=1.2)
    _, _, v = W.make_qkv(w)
    say("mask -> forward")
    indptr, indices = gpu_mask(w, q, k, 0.9)
    prob = Problem(w, q, k, v, mask=(indptr, indices))
    p = prob.params()
    assert F.fgattn_validate_mask(prob.d_indptr, prob.d_indices, p, prob.workspace(p)) == 0
    got = prob.run()
    check_against_oracle(oracle_mod, prob, got, what=w.name)


@pytest.mark.parametrize("flags", [0, F.FLAG_MASK_ROWS_IN_HBM], ids=["bins-in-lds", "rows-in-hbm"])
def test_p_one_keeps_what_the_fixed_point_resolves(oracle_mod, flags):
    # top_p = 1 on peaked rows: weights are 2^-40 fixed point relative to the row maximum, so a key block more than
    # 40 ln 2 = 27.7 below the maximum weighs nothing and is dropped (all of them together hold less than G * 2^-40
    # of the mass); the fp64 oracle keeps every key block.  Everything within 27 of the maximum must be kept,
    # nothing further than 27.8 below it may be.
    w = W.Workload("mask-p-one-peaked", H=2, L=3000, d=64, M=32, N=1, grid=(1, 1, 3000), seed=4700)
    q, k = W.make_qk_local(w, gain=3.0, bandwidth=0.02)
    say("mask p = 1, peaked rows, flags=%d" % flags)
    indptr, indices = gpu_mask(w, q, k, 1.0, flags=flags)
    rows = list(range(w.items))
    ref = oracle_mod.topp_rows(q, k, w.M, w.N, float(np.float32(w.scale)), 1.0, rows=rows)
    dropped_somewhere = 0
    for row, (kept, order, cum) in zip(rows, ref):
        prob = np.empty(w.G)
        prob[order] = np.diff(np.concatenate([[0.0], cum]))
        below_max = np.log(prob.max()) - np.log(np.maximum(prob, 1e-300))   # score distance to the row maximum
        inside = np.zeros(w.G, dtype=bool)
        inside[indices[indptr[row]:indptr[row + 1]]] = True
        assert inside[below_max <= 27.0].all(), "row %d: a key block with weight was dropped" % row
        assert not inside[below_max >= 27.8].any(), "row %d: a key block without weight was kept" % row
        assert prob[~inside].sum() < w.G * 2.0 ** -40
        dropped_somewhere += int((~inside).any())
    say("    %d of %d rows drop weightless key blocks" % (dropped_somewhere, w.items))
    assert dropped_somewhere > 0, "the inputs were meant to have rows with key blocks below the resolution"


def test_emit_with_too_small_a_capacity_drops_the_tail():
    # a caller that passes fewer entries than the mask holds gets the leading entries and no write past them
    w = W.Workload("mask-short-capacity", H=2, L=2048, d=64, M=32, N=1, grid=(8, 16, 16), seed=4600)
    q, k = W.make_qk_local(w, gain=1.5)
    indptr, indices = gpu_mask(w, q, k, 0.9)
    dq, dk = to_dev_bf16(q), to_dev_bf16(k)
    p = F.make_params(dq, dk, dk, dq, w.M, w.N, w.scale)
    ws = torch.empty(F.fgattn_mask_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    d_indptr = torch.empty(w.items + 1, dtype=torch.int64, device="cuda")
    F.fgattn_mask_select(dq, dk, p, 0.9, d_indptr, ws)
    nnz = indices.size
    for cap in (nnz - 1, nnz // 2, 1, 0):
        buf = torch.full((nnz + 8,), -7, dtype=torch.int32, device="cuda")
        F.fgattn_mask_emit(p, d_indptr, buf[:cap], ws)
        torch.cuda.synchronize()
        got = buf.cpu().numpy()
        assert np.array_equal(got[:cap], indices[:cap]) and (got[cap:] == -7).all(), cap


def test_mask_argument_checks():
    w = W.TINY
    q, k, _ = W.make_qkv(w)
    dq, dk = to_dev_bf16(q), to_dev_bf16(k)
    p = F.make_params(dq, dk, dk, dq, w.M, w.N, w.scale)
    ws = torch.empty(F.fgattn_mask_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    indptr = torch.zeros(w.items + 1, dtype=torch.int64, device="cuda")
    for bad_p in (0.0, -0.1, 1.5, float("nan")):
        with pytest.raises(F.FgattnError) as e:
            F.fgattn_mask_select(dq, dk, p, bad_p, indptr, ws)
        assert e.value.code == F.E_SCALE
    with pytest.raises(F.FgattnError) as e:
        F.fgattn_mask_select(dq, dk, p, 0.9, indptr, ws[:1024])
    assert e.value.code == F.E_WORKSPACE
    p2 = F.make_params(dq, dk, dk, dq, 48, w.N, w.scale)
    assert F.fgattn_mask_workspace_bytes(p2) == 0


def test_mask_full_size_wan(oracle_mod):
    # config-2 shape: 6144 query blocks x 32760 key blocks; sampled rows against the oracle, all rows by properties
    w = W.WAN_1_3B
    q, k = W.make_qk_local(w, gain=1.0)
    say("mask wan-1.3b p=0.9")
    indptr, indices = gpu_mask(w, q, k, 0.9)
    nnz = np.diff(indptr)
    say("    density %.3f, per block min %d max %d" % (indices.size / float(w.items * w.G), nnz.min(), nnz.max()))
    d_indptr, d_indices = torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda()
    dq = to_dev_bf16(q)
    p = F.make_params(dq, dq, dq, dq, w.M, w.N, w.scale)
    ws = torch.empty(F.fgattn_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    assert F.fgattn_validate_mask(d_indptr, d_indices, p, ws) == 0
    rng = np.random.default_rng(0)
    rows = sorted({0, w.QB - 1, w.items - 1, int(np.argmax(nnz)), int(np.argmin(nnz))} |
                  set(rng.choice(w.items, size=43, replace=False).tolist()))
    bad = check_rows(oracle_mod, w, q, k, 0.9, indptr, indices, rows, what=w.name)


def test_mask_full_size_hunyuan(oracle_mod):
    # config-4 shape: 22296 query blocks x 118800 key blocks (10.6 GB of scores, passed through a 1 GiB buffer in
    # eleven chunks); rows this long are selected from device memory.  Sampled rows against the oracle, all rows
    # by the validator.
    w = W.HUNYUAN
    q, k = W.make_qk_local(w, gain=2.5)
    say("mask hunyuan p=0.9")
    indptr, indices = gpu_mask(w, q, k, 0.9)
    nnz = np.diff(indptr)
    say("    density %.3f, per block min %d max %d" % (indices.size / float(w.items * w.G), nnz.min(), nnz.max()))
    d_indptr, d_indices = torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda()
    dq = to_dev_bf16(q)
    p = F.make_params(dq, dq, dq, dq, w.M, w.N, w.scale)
    ws = torch.empty(F.fgattn_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    assert F.fgattn_validate_mask(d_indptr, d_indices, p, ws) == 0
    rng = np.random.default_rng(1)
    # the score buffer holds 17 tiles of 128 query blocks (8 tiles per head, the last one with 33 used rows): the
    # last row of the first chunk and the first of the second, and the two sides of a head's short last tile
    tiles_per_head = -(-w.QB // 128)
    assert tiles_per_head == 8 and (1 << 30) // (128 * 118816 * 4) == 17
    edge = [2 * w.QB + 127, 2 * w.QB + 128, w.QB - 1, w.QB, 7 * 128 - 1, 7 * 128]
    rows = sorted({0, w.items - 1, int(np.argmax(nnz)), int(np.argmin(nnz))} | set(edge) |
                  set(rng.choice(w.items, size=8, replace=False).tolist()))
    bad = check_rows(oracle_mod, w, q, k, 0.9, indptr, indices, rows, what=w.name)


def _random_mask_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for c in range(n):
        M = int(rng.choice([16, 32, 64, 128]))
        d = int(rng.choice([64, 128]))
        N = int(rng.choice([1, 1, 2, 3, 8, 17, 32, 64]))
        L = int(rng.integers(8, 2500))
        H = int(rng.integers(1, 4))
        top_p = float(rng.choice([0.3, 0.7, 0.9, 0.99]))
        gain = float(rng.choice([0.0, 1.0, 2.0]))
        cases.append((M, N, d, L, H, top_p, gain, 4700 + c))
    return cases


@pytest.mark.parametrize("M,N,d,L,H,top_p,gain,seed", _random_mask_cases(16, 20250928))
def test_mask_seeded_random_shapes(oracle_mod, M, N, d, L, H, top_p, gain, seed):
    # shapes nobody picked by hand, drawn from a fixed seed; every query block against the oracle
    w = W.Workload("mask-rand-M%d-N%d-d%d-L%d" % (M, N, d, L), H=H, L=L, d=d, M=M, N=N, grid=(1, 1, L), seed=seed)
    if gain > 0.0:
        q, k = W.make_qk_local(w, gain=gain, bandwidth=0.02)
    else:
        q, k, _ = W.make_qkv(w)
    say("mask %s H=%d p=%.2f gain=%.1f" % (w.name, H, top_p, gain))
    indptr, indices, pooled = gpu_mask(w, q, k, top_p, want_pooled=True)
    assert np.array_equal(pooled, oracle_mod.pool(q, M)), "query block means differ from the oracle's bits"
    bad = check_rows(oracle_mod, w, q, k, top_p, indptr, indices, list(range(w.items)), what=w.name)


@pytest.mark.parametrize("M,N,L,top_p", [(64, 64, 8, 0.9), (16, 128, 130, 0.5), (128, 1, 1, 1.0), (32, 1, 2, 0.99), (16, 1, 33, 1.0)])
def test_mask_degenerate_sizes(oracle_mod, M, N, L, top_p):
    # one or two key blocks, a single token, fewer tokens than one query block, p = 1
    w = W.Workload("mask-degenerate-M%d-N%d-L%d" % (M, N, L), H=2, L=L, d=64, M=M, N=N, seed=4900 + L)
    q, k, _ = W.make_qkv(w)
    say("mask %s p=%.2f" % (w.name, top_p))
    indptr, indices = gpu_mask(w, q, k, top_p)
    check_rows(oracle_mod, w, q, k, top_p, indptr, indices, list(range(w.items)), what=w.name)


def _wide_random_mask_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for c in range(n):
        M = int(rng.choice([16, 32, 64, 128]))
        d = int(rng.choice([64, 128]))
        N = int(rng.choice([1, 1, 1, 2, 3, 8, 17, 32, 64]))
        L = int(rng.integers(1, 6000))
        H = int(rng.integers(1, 5))
        top_p = float(rng.choice([0.1, 0.3, 0.5, 0.7, 0.9, 0.99]))
        gain = float(rng.choice([0.0, 1.0, 2.0, 3.0]))
        flags = int(rng.choice([0, 0, 8, 16, 24]))
        cases.append((M, N, d, L, H, top_p, gain, flags, 15000 + c))
    return cases


@pytest.mark.parametrize("M,N,d,L,H,top_p,gain,flags,seed", _wide_random_mask_cases(48, 20251129))
def test_mask_seeded_random_shapes_wide(oracle_mod, M, N, d, L, H, top_p, gain, flags, seed):
    # a wider draw than test_mask_seeded_random_shapes: longer sequences, more values of p, both selection kernels and
    # the one-tile score buffer; every query block against the oracle (sampled ones where that is too many scores)
    w = W.Workload("mask-wide-M%d-N%d-d%d-L%d-s%d" % (M, N, d, L, seed), H=H, L=L, d=d, M=M, N=N, grid=(1, 1, L), seed=seed)
    if gain > 0.0:
        q, k = W.make_qk_local(w, gain=gain, bandwidth=0.02)
    else:
        q, k, _ = W.make_qkv(w)
    say("mask %s H=%d p=%.2f gain=%.1f flags=%d" % (w.name, H, top_p, gain, flags))
    indptr, indices = gpu_mask(w, q, k, top_p, flags=flags)
    rows = list(range(w.items))
    if w.items * w.G > 3e6:
        rows = sorted(set(np.random.default_rng(seed).integers(0, w.items, size=20).tolist()) | {0, w.items - 1})
    check_rows(oracle_mod, w, q, k, top_p, indptr, indices, rows, what=w.name)
