"""Error behaviour of the C ABI on a GPU machine: bad arguments come back as codes, nothing is launched."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2509_16518_amd import fgattn as F
from paper_2509_16518_amd import workloads as W
from gpu_util import Problem

pytestmark = pytest.mark.gpu


def expect(code, fn):
    with pytest.raises(F.FgattnError) as e:
        fn()
    assert e.value.code == code, (e.value.code, code)


def test_argument_errors():
    prob = Problem(W.TINY)
    p = prob.params()
    ws = prob.workspace(p)
    call = lambda pp, w=ws, q=None: F.fgattn_forward(q if q is not None else prob.q, prob.k, prob.v, prob.d_indptr,
                                                     prob.d_indices, pp, prob.out, prob.lse, w)
    bad = prob.params(); bad.d = 96
    expect(F.E_SHAPE, lambda: call(bad))
    bad = prob.params(); bad.M = 48
    expect(F.E_SHAPE, lambda: call(bad))
    bad = prob.params(); bad.N = 0
    expect(F.E_SHAPE, lambda: call(bad))
    bad = prob.params(); bad.q_stride_l = 60
    expect(F.E_STRIDE, lambda: call(bad))
    bad = prob.params(); bad.scale = float("inf")
    expect(F.E_SCALE, lambda: call(bad))
    bad = prob.params(); bad.flags = 64
    expect(F.E_FLAGS, lambda: call(bad))
    expect(F.E_WORKSPACE, lambda: call(p, ws[:256]))
    expect(F.E_ALIGN, lambda: call(p, ws[16:]))
    qoff = prob.q.view(-1)[4:]                                  # 8-byte offset: not 16-byte aligned
    rc = F.lib().fgattn_forward(qoff.data_ptr(), prob.k.data_ptr(), prob.v.data_ptr(), prob.d_indptr.data_ptr(),
                                prob.d_indices.data_ptr(), ctypes.byref(p), prob.out.data_ptr(), prob.lse.data_ptr(),
                                ws.data_ptr(), ws.numel(), None)
    assert rc == F.E_ALIGN
    assert F.lib().fgattn_forward(None, None, None, None, None, None, None, None, None, 0, None) == F.E_NULL
    assert "workspace" in F.fgattn_strerror(F.E_WORKSPACE)


def test_validate_mask_flags_bad_masks():
    prob = Problem(W.TINY)
    p = prob.params()
    ws = prob.workspace(p)
    assert F.fgattn_validate_mask(prob.d_indptr, prob.d_indices, p, ws) == 0
    dup = prob.d_indices.clone(); dup[1] = dup[0]
    assert F.fgattn_validate_mask(prob.d_indptr, dup, p, ws) == F.E_MASK
    oob = prob.d_indices.clone(); oob[5] = prob.w.G
    assert F.fgattn_validate_mask(prob.d_indptr, oob, p, ws) == F.E_MASK
    neg = prob.d_indices.clone(); neg[7] = -1
    assert F.fgattn_validate_mask(prob.d_indptr, neg, p, ws) == F.E_MASK
    dec = prob.d_indptr.clone(); dec[3] = dec[2] - 1
    assert F.fgattn_validate_mask(dec, prob.d_indices, p, ws) == F.E_MASK


@pytest.mark.parametrize("M", [64, 128])
def test_forward_part_is_a_measurement_aid_only(M):
    # built for M = 64 / 128, d = 128, N = 1 only; runs, leaves the real entry point's results untouched afterwards
    w = W.Workload("part", H=2, L=2048, d=128, M=M, N=1, kind=W.MASK_RANDOM, density=0.3, seed=5100)
    prob = Problem(w)
    p = prob.params(flags=F.FLAG_REUSE_PLAN)
    ws = prob.workspace(p)
    F.fgattn_plan(prob.d_indptr, p, ws)
    scratch_out, scratch_lse = torch.empty_like(prob.out), torch.empty_like(prob.lse)
    parts = (F.PART_GATHER, F.PART_COMPUTE) + ((F.PART_GATHER_RING3, F.PART_GATHER_ONE_WG) if M == 64 else ())
    for part in parts:
        F.fgattn_forward_part(prob.q, prob.k, prob.v, prob.d_indptr, prob.d_indices, p, scratch_out, scratch_lse, ws, part)
    torch.cuda.synchronize()
    for bad in (0, 5):
        expect(F.E_FLAGS, lambda: F.fgattn_forward_part(prob.q, prob.k, prob.v, prob.d_indptr, prob.d_indices, p, scratch_out,
                                                        scratch_lse, ws, bad))
    if M == 128:   # the ring / occupancy variants of the gather half are built for the 64-row tile only
        expect(F.E_SHAPE, lambda: F.fgattn_forward_part(prob.q, prob.k, prob.v, prob.d_indptr, prob.d_indices, p, scratch_out,
                                                        scratch_lse, ws, F.PART_GATHER_RING3))
    tiny = Problem(W.TINY)
    pt = tiny.params()
    expect(F.E_SHAPE, lambda: F.fgattn_forward_part(tiny.q, tiny.k, tiny.v, tiny.d_indptr, tiny.d_indices, pt, tiny.out,
                                                    tiny.lse, tiny.workspace(pt), F.PART_GATHER))
    # the stored order is still usable: the partial kernels rewind the queue like the full one
    F.fgattn_forward(prob.q, prob.k, prob.v, prob.d_indptr, prob.d_indices, p, prob.out, prob.lse, ws)
    torch.cuda.synchronize()
    a = prob.out.clone()
    got = prob.run()
    assert torch.equal(a, prob.out)


def test_issue_probe_is_a_measurement_aid_only():
    # runs for the instruction mixes it is built for, touches only its scratch, rejects everything else
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    scratch = torch.zeros(2048 * cus + 64, dtype=torch.uint8, device="cuda")
    scratch[2048 * cus:] = 0x5A
    for other in (0, 59, 61, 67):
        flop = F.fgattn_issue_probe(other, 8, scratch[:2048 * cus])
        assert flop == 2.0 * cus * 4 * 8 * 16 * 32768.0
    torch.cuda.synchronize()
    assert bool((scratch[2048 * cus:] == 0x5A).all())
    expect(F.E_FLAGS, lambda: F.fgattn_issue_probe(7, 8, scratch))
    expect(F.E_WORKSPACE, lambda: F.fgattn_issue_probe(67, 8, scratch[:1024]))
    expect(F.E_SHAPE, lambda: F.fgattn_issue_probe(67, 0, scratch))


@pytest.mark.parametrize("M,N,L", [(64, 1, 32760), (128, 32, 32760), (128, 32, 32768), (16, 8, 1000)])
def test_grid_size_is_reported_for_every_variant(M, N, L):
    q = torch.empty((1, 2, L, 128), dtype=torch.bfloat16, device="cuda")
    p = F.make_params(q, q, q, q, M, N, 0.1)
    grid = F.lib().fgattn_grid_size(ctypes.byref(p))
    assert 1 <= grid <= 4096


def test_forward_is_graph_capturable():
    # the library allocates nothing and clears no memory on the hot path: a call (ordering pre-pass + kernel) can be
    # captured into a graph; every replay must reproduce the eager result bit for bit
    w = W.Workload("graph", H=3, L=2048, d=128, M=64, N=1, kind=W.MASK_SKEW_LEN, density=0.3, skew=0.7, seed=5200)
    prob = Problem(w)
    p = prob.params()
    ws = prob.workspace(p)
    F.fgattn_forward(prob.q, prob.k, prob.v, prob.d_indptr, prob.d_indices, p, prob.out, prob.lse, ws)   # also warms caches
    torch.cuda.synchronize()
    ref_out, ref_lse = prob.out.clone(), prob.lse.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        F.fgattn_forward(prob.q, prob.k, prob.v, prob.d_indptr, prob.d_indices, p, prob.out, prob.lse, ws)
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            F.fgattn_forward(prob.q, prob.k, prob.v, prob.d_indptr, prob.d_indices, p, prob.out, prob.lse, ws)
    torch.cuda.synchronize()
    for replay in range(3):
        prob.out.view(torch.int16).fill_(0x7FC0)
        prob.lse.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(prob.out.view(torch.int16), ref_out.view(torch.int16)), "replay %d: out differs" % replay
        assert torch.equal(prob.lse, ref_lse), "replay %d: lse differs" % replay
        # eager work between the replays
        F.fgattn_forward(prob.q, prob.k, prob.v, prob.d_indptr, prob.d_indices, p, prob.out, prob.lse, ws)
        torch.cuda.synchronize()
        assert torch.equal(prob.out.view(torch.int16), ref_out.view(torch.int16))
