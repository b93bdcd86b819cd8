"""GPU parity of the grouped-query-tile forward pass (paper Sec. 4.2) through the C ABI.

Grouping changes what is LOADED (the union of the members' key lists), never what is attended: the reference is
the attention oracle on the original, ungrouped mask.  The groupings themselves come from the grouping oracle
(merge-consecutive and greedy merge-XOR) or, further down, from the GPU pre-pass, which must reproduce them exactly.
"""
import numpy as np
import pytest
import torch

from oracle import grouping as GR
from paper_2509_16518_amd import fgattn as F
from paper_2509_16518_amd import workloads as W
from gpu_util import Problem, check_against_oracle, say

pytestmark = pytest.mark.gpu


def run_grouped(prob, tiles, up, ui, um):
    w = prob.w
    p = prob.params()
    ws = prob.workspace(p)
    d_tiles = torch.from_numpy(np.ascontiguousarray(tiles.reshape(-1))).cuda()
    d_up = torch.from_numpy(up).cuda()
    d_ui = torch.from_numpy(ui if ui.size else np.zeros(1, np.int32)).cuda()
    d_um = torch.from_numpy(um if um.size else np.zeros(1, np.uint8)).cuda()
    prob.out.view(torch.int16).fill_(0x7FC0)
    prob.lse.fill_(float("nan"))
    F.fgattn_forward_grouped(prob.q, prob.k, prob.v, d_tiles, d_up, d_ui, d_um, p, prob.out, prob.lse, ws)
    torch.cuda.synchronize()
    from gpu_util import out_to_f64
    return out_to_f64(prob.out), prob.lse.double().cpu().numpy()


@pytest.mark.parametrize("mode", ["consecutive", "xor"])
@pytest.mark.parametrize("M,N,d,L", [(32, 1, 128, 1024), (16, 1, 64, 1024), (64, 8, 128, 1024), (16, 8, 128, 1000),
                                     (32, 3, 64, 1000), (64, 1, 64, 1000), (128, 1, 128, 1024)])
def test_grouped_matches_oracle_on_the_ungrouped_mask(oracle_mod, mode, M, N, d, L):
    w = W.Workload("grouped-%s-M%d-N%d-d%d-L%d" % (mode, M, N, d, L), H=2, L=L, d=d, M=M, N=N, kind=W.MASK_RANDOM,
                   density=0.3, seed=6000 + M + N)
    prob = Problem(w)
    R = 128 // M
    say("grouped %s" % w.name)
    tiles, up, ui, um = GR.grouped_mask(prob.indptr, prob.indices, w.H, w.QB, w.G, R, mode)
    got = run_grouped(prob, tiles, up, ui, um)
    check_against_oracle(oracle_mod, prob, got, what=w.name)
    say("    union entries %d vs %d in the tiles' own lists" % (ui.size, prob.indices.size))


def test_grouped_with_empty_members_and_repeating_patterns(oracle_mod):
    # tiles repeat three key patterns (one of them empty): merge-XOR puts equal patterns together, so a group's union
    # is one pattern; merge-consecutive mixes them.  Both must give the ungrouped result.
    w = W.Workload("grouped-patterns", H=2, L=1536, d=128, M=32, N=4, seed=6100)
    rng = np.random.default_rng(5)
    pats = [np.sort(rng.choice(w.G, size=n, replace=False)).astype(np.int32) for n in (90, 60)] + [np.zeros(0, np.int32)]
    rows = [pats[(i + s) % 3] for s in range(w.H) for i in range(w.QB)]
    indptr = np.zeros(len(rows) + 1, np.int64)
    indptr[1:] = np.cumsum([r.size for r in rows])
    prob = Problem(w, mask=(indptr, np.concatenate(rows)))
    for mode in ("xor", "consecutive"):
        tiles, up, ui, um = GR.grouped_mask(prob.indptr, prob.indices, w.H, w.QB, w.G, 4, mode)
        say("grouped patterns %s: union entries %d" % (mode, ui.size))
        got = run_grouped(prob, tiles, up, ui, um)
        check_against_oracle(oracle_mod, prob, got, what=w.name + " " + mode)


def gpu_grouping(prob, mode):
    """Runs the device pre-pass; returns (tiles [groups, R], union_indptr, union_indices, union_members) as numpy."""
    w = prob.w
    p = prob.params()
    R = 128 // w.M
    NG = (w.QB + R - 1) // R
    groups = w.B * w.H * NG
    m = F.GROUP_XOR if mode == "xor" else F.GROUP_CONSECUTIVE
    ws = torch.empty(F.fgattn_group_workspace_bytes(p, m), dtype=torch.uint8, device="cuda")
    tiles = torch.full((groups * R,), -9, dtype=torch.int32, device="cuda")
    up = torch.full((groups + 1,), -1, dtype=torch.int64, device="cuda")
    F.fgattn_group_select(prob.d_indptr, prob.d_indices, p, m, tiles, up, ws)
    nnz = int(up[-1].item())
    ui = torch.full((nnz + 8,), -7, dtype=torch.int32, device="cuda")
    um = torch.full((nnz + 8,), 0xEE, dtype=torch.uint8, device="cuda")
    F.fgattn_group_emit(p, m, tiles, up, ui[:nnz], um[:nnz], ws)
    torch.cuda.synchronize()
    assert (ui[nnz:] == -7).all() and (um[nnz:] == 0xEE).all(), "emit wrote past the capacity"
    return tiles.cpu().numpy().reshape(groups, R), up.cpu().numpy(), ui[:nnz].cpu().numpy(), um[:nnz].cpu().numpy()


@pytest.mark.parametrize("mode", ["consecutive", "xor"])
@pytest.mark.parametrize("M,N,L,kind", [(32, 1, 1024, W.MASK_RANDOM), (16, 8, 1000, W.MASK_WINDOW_FILL), (64, 3, 1000, W.MASK_RANDOM),
                                        (16, 1, 3000, W.MASK_WINDOW_FILL)])
def test_device_grouping_equals_the_oracles(mode, M, N, L, kind):
    grid = {1024: (4, 16, 16), 1000: (10, 10, 10), 3000: (3, 25, 40)}[L]
    w = W.Workload("grouping-%s-M%d-N%d-L%d" % (mode, M, N, L), H=3, L=L, d=64, M=M, N=N, grid=grid, window=(1, 2, 2),
                   kind=kind, density=0.3, seed=6200 + M + N)
    prob = Problem(w)
    say("device grouping %s" % w.name)
    got = gpu_grouping(prob, mode)
    ref = GR.grouped_mask(prob.indptr, prob.indices, w.H, w.QB, w.G, 128 // M, mode)
    for a, b, name in zip(got, ref, ("group_tiles", "union_indptr", "union_indices", "union_members")):
        assert np.array_equal(a, b), name


def test_device_grouping_many_tiles():
    # 4688 tiles per slice: more than the register-resident variant of the greedy pre-pass takes
    w = W.Workload("grouping-many-tiles", H=1, L=75000, d=64, M=16, N=64, kind=W.MASK_RANDOM, density=0.3, seed=6500)
    prob = Problem(w)
    say("device grouping %s: %d tiles, %d key blocks" % (w.name, w.QB, w.G))
    got = gpu_grouping(prob, "xor")
    ref = GR.grouped_mask(prob.indptr, prob.indices, w.H, w.QB, w.G, 8, "xor")
    for a, b, name in zip(got, ref, ("group_tiles", "union_indptr", "union_indices", "union_members")):
        assert np.array_equal(a, b), name


def test_device_grouping_then_forward(oracle_mod):
    # everything on the device: mask -> grouping -> grouped attention, against the oracle on the ungrouped mask
    w = W.Workload("group-then-attend", H=2, L=2048, d=128, M=32, N=1, grid=(8, 16, 16), window=(1, 3, 3),
                   kind=W.MASK_WINDOW_FILL, density=0.3, seed=6300)
    prob = Problem(w)
    for mode in ("xor", "consecutive"):
        tiles, up, ui, um = gpu_grouping(prob, mode)
        say("device grouping + forward %s: union entries %d vs %d" % (mode, ui.size, prob.indices.size))
        got = run_grouped(prob, tiles, up, ui, um)
        check_against_oracle(oracle_mod, prob, got, what=w.name + " " + mode)


def test_device_grouping_with_batch(oracle_mod):
    # B = 2: slices are (batch, head) pairs; ragged last tile and last group (1000 = 31 * 32 + 8; 32 tiles = 8 groups)
    import dataclasses
    w = dataclasses.replace(W.Workload("group-batch", H=2, L=1000, d=64, M=32, N=1, grid=(10, 10, 10), window=(1, 2, 2),
                                       kind=W.MASK_WINDOW_FILL, density=0.3, seed=6400), B=2)
    prob = Problem(w)
    for mode in ("xor", "consecutive"):
        got = gpu_grouping(prob, mode)
        ref = GR.grouped_mask(prob.indptr, prob.indices, w.B * w.H, w.QB, w.G, 4, mode)
        for a, b, name in zip(got, ref, ("group_tiles", "union_indptr", "union_indices", "union_members")):
            assert np.array_equal(a, b), name + " " + mode
        say("device grouping B=2 %s: union entries %d" % (mode, got[2].size))
        out = run_grouped(prob, *got)
        check_against_oracle(oracle_mod, prob, out, what=w.name + " " + mode)


@pytest.mark.parametrize("M,N,L", [(16, 1, 40), (16, 1, 16), (32, 8, 33), (64, 1, 200)])
def test_device_grouping_degenerate_sizes(oracle_mod, M, N, L):
    # fewer tiles than a group holds, a single tile, a single-row last tile, one group per slice plus a remainder
    w = W.Workload("group-degenerate-M%d-N%d-L%d" % (M, N, L), H=2, L=L, d=64, M=M, N=N, kind=W.MASK_RANDOM,
                   density=0.5, seed=6600 + L)
    prob = Problem(w)
    for mode in ("xor", "consecutive"):
        got = gpu_grouping(prob, mode)
        ref = GR.grouped_mask(prob.indptr, prob.indices, w.H, w.QB, w.G, 128 // M, mode)
        for a, b, name in zip(got, ref, ("group_tiles", "union_indptr", "union_indices", "union_members")):
            assert np.array_equal(a, b), name + " " + mode
        out = run_grouped(prob, *got)
        check_against_oracle(oracle_mod, prob, out, what=w.name + " " + mode)


def test_grouping_argument_checks():
    prob = Problem(W.TINY)
    p = prob.params()
    assert F.fgattn_group_workspace_bytes(p, 7) == 0
    ws = torch.empty(F.fgattn_group_workspace_bytes(p, F.GROUP_XOR), dtype=torch.uint8, device="cuda")
    tiles = torch.empty(prob.w.items, dtype=torch.int32, device="cuda")
    up = torch.empty(prob.w.items // 8 + 1, dtype=torch.int64, device="cuda")
    with pytest.raises(F.FgattnError) as e:
        F.fgattn_group_select(prob.d_indptr, prob.d_indices, p, 7, tiles, up, ws)
    assert e.value.code == F.E_FLAGS
    with pytest.raises(F.FgattnError) as e:
        F.fgattn_group_select(prob.d_indptr, prob.d_indices, p, F.GROUP_XOR, tiles, up, ws[:512])
    assert e.value.code == F.E_WORKSPACE


def _random_group_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for c in range(n):
        M = int(rng.choice([16, 32, 64]))
        d = int(rng.choice([64, 128]))
        N = int(rng.choice([1, 1, 2, 3, 8, 16, 32, 64]))
        L = int(rng.integers(1, 4000))
        H = int(rng.integers(1, 4))
        B = int(rng.choice([1, 1, 2]))
        kind = [W.MASK_RANDOM, W.MASK_SKEW_LEN, W.MASK_WINDOW_FILL][int(rng.integers(0, 3))]
        density = float(rng.choice([0.05, 0.3, 0.6]))
        mode = ["consecutive", "xor"][int(rng.integers(0, 2))]
        cases.append((M, N, d, L, H, B, kind, density, mode, 6700 + c))
    return cases


@pytest.mark.parametrize("M,N,d,L,H,B,kind,density,mode,seed", _random_group_cases(32, 20251130))
def test_grouping_seeded_random_shapes(oracle_mod, M, N, d, L, H, B, kind, density, mode, seed):
    # shapes nobody picked by hand: the device pre-pass must equal the grouping oracle bit for bit, and the grouped
    # forward pass on its output must agree with the attention oracle on the UNGROUPED mask
    import dataclasses
    w = W.Workload("group-rand-M%d-N%d-d%d-L%d" % (M, N, d, L), H=H, L=L, d=d, M=M, N=N, grid=(1, 1, L), window=(0, 0, 9),
                   kind=kind, density=density, seed=seed, skew=0.7)
    w = dataclasses.replace(w, B=B)
    prob = Problem(w)
    say("grouping random %s H=%d B=%d kind=%d density=%.2f %s" % (w.name, H, B, kind, density, mode))
    got = gpu_grouping(prob, mode)
    ref = GR.grouped_mask(prob.indptr, prob.indices, w.B * w.H, w.QB, w.G, 128 // M, mode)
    for a, b, name in zip(got, ref, ("group_tiles", "union_indptr", "union_indices", "union_members")):
        assert np.array_equal(a, b), name
    out = run_grouped(prob, *got)
    check_against_oracle(oracle_mod, prob, out, what=w.name + " " + mode)
