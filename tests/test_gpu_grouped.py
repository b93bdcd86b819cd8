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
