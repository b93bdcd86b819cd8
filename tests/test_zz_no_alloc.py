"""The entry point that allocates nothing (fgattn_forward_static: scratch inside the library's device image)
against fgattn_forward on the same inputs, through the C ABI: two calls in a row, the second on a smaller input
(the scratch keeps the first call's contents), plus the size limit."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2509_16518_amd import fgattn as F
from paper_2509_16518_amd import workloads as W
from gpu_util import Problem, check_against_oracle, out_to_f64, say

pytestmark = pytest.mark.gpu


def run_static(prob, flags=0):
    p = prob.params(flags=flags)
    prob.out.view(torch.int16).fill_(0x7FC0)
    prob.lse.fill_(float("nan"))
    F.fgattn_forward_static(prob.q, prob.k, prob.v, prob.d_indptr, prob.d_indices, p, prob.out, prob.lse)
    torch.cuda.synchronize()
    return out_to_f64(prob.out), prob.lse.double().cpu().numpy()


def same(a, b):
    return np.array_equal(a, b, equal_nan=True)


def test_static_entry_point_matches_forward_twice(oracle_mod):
    big = W.Workload("static-big", H=6, L=3000, d=128, M=64, N=1, grid=(3, 25, 40), window=(1, 3, 3), seed=7100)
    small = W.Workload("static-small", H=2, L=1000, d=64, M=16, N=8, grid=(10, 10, 10), window=(1, 2, 2), seed=7101)
    for n, w in enumerate((big, small)):
        say("static entry point, call %d: %s (%d work items)" % (n + 1, w.name, w.items))
        prob = Problem(w)
        ref = prob.run()                       # fgattn_forward with a caller workspace
        got = run_static(prob)
        # same kernels, same order of work: the two entry points agree bit for bit (and with the oracle to the bar)
        assert same(got[0], ref[0]) and same(got[1], ref[1]), w.name
        check_against_oracle(oracle_mod, prob, got, what=w.name)
        # the order left in the scratch by the call above is reusable by the next call of this entry point
        again = run_static(prob, flags=F.FLAG_REUSE_PLAN)
        assert same(again[0], ref[0]) and same(again[1], ref[1]), w.name + " (reused plan)"


def test_static_entry_point_rejects_too_many_items():
    w = W.Workload("static-limit", H=1, L=256, d=64, M=16, N=1, seed=7102)
    prob = Problem(w, mask=(np.zeros(w.items + 1, np.int64), np.zeros(0, np.int32)))
    p = prob.params()
    p.H = F.STATIC_MAX_ITEMS // w.QB + 1            # more work items than the scratch holds: refused before any launch
    rc = F.lib().fgattn_forward_static(prob.q.data_ptr(), prob.k.data_ptr(), prob.v.data_ptr(), prob.d_indptr.data_ptr(),
                                       prob.d_indices.data_ptr(), ctypes.byref(p), prob.out.data_ptr(),
                                       prob.lse.data_ptr(), None)
    assert rc == F.E_STATIC_LIMIT and "STATIC_MAX_ITEMS" in F.fgattn_strerror(rc)
    p.H = F.STATIC_MAX_ITEMS // w.QB                # exactly at the limit the shape check passes (H * QB == max)
    assert p.H * w.QB == F.STATIC_MAX_ITEMS
