"""Helpers for the GPU parity tests: upload a workload, run the HIP path through the C ABI, compare."""
import numpy as np
import torch

from paper_2509_16518_amd import fgattn as F
from paper_2509_16518_amd import workloads as W

# Tolerances fixed by the benchmark spec for bf16 inputs: out max-abs <= 2e-2, mean-abs <= 2e-3,
# lse within 1e-3 relative (taken as |d| <= 1e-3 * max(1, |lse|), since a relative bound is
# ill-conditioned near lse = 0).
OUT_MAX_ABS = 2e-2
OUT_MEAN_ABS = 2e-3
LSE_REL = 1e-3


def say(msg):
    print(msg, flush=True)


def to_dev_bf16(bits):
    """uint16 bf16 bit patterns (numpy) -> torch.bfloat16 tensor on the GPU, same bits."""
    t = torch.from_numpy(bits.view(np.int16)).cuda()
    return t.view(torch.bfloat16)


def out_to_f64(out):
    """bf16 device tensor -> float64 numpy (exact widening)."""
    return W.bf16_bits_to_f64(out.view(torch.int16).cpu().numpy().view(np.uint16))


class Problem:
    """Device-resident tensors and mask of one workload."""

    def __init__(self, w, q_bits=None, k_bits=None, v_bits=None, mask=None):
        self.w = w
        if q_bits is None:
            q_bits, k_bits, v_bits = W.make_qkv(w)
        self.q_bits, self.k_bits, self.v_bits = q_bits, k_bits, v_bits
        self.indptr, self.indices = mask if mask is not None else W.make_mask(w)
        self.q, self.k, self.v = (to_dev_bf16(x) for x in (q_bits, k_bits, v_bits))
        self.d_indptr = torch.from_numpy(self.indptr).cuda()
        # keep at least one element so data_ptr() is a valid device pointer even for an empty mask
        self.d_indices = torch.from_numpy(self.indices if self.indices.size else np.zeros(1, np.int32)).cuda()
        self.out = torch.empty_like(self.q)
        self.lse = torch.empty(self.q.shape[:3], dtype=torch.float32, device="cuda")

    def params(self, scale=None, flags=0, q=None, k=None, v=None, out=None):
        w = self.w
        return F.make_params(q if q is not None else self.q, k if k is not None else self.k,
                             v if v is not None else self.v, out if out is not None else self.out,
                             w.M, w.N, w.scale if scale is None else scale, flags)

    def workspace(self, p):
        n = F.fgattn_workspace_bytes(p)
        assert n > 0
        return torch.empty(n, dtype=torch.uint8, device="cuda")

    def run(self, scale=None, flags=0, dense=False, poison=True):
        """One forward call; returns (out float64 [B,H,L,d], lse float64 [B,H,L])."""
        p = self.params(scale, flags)
        ws = self.workspace(p)
        if poison:
            self.out.view(torch.int16).fill_(0x7FC0)  # bf16 NaN
            self.lse.fill_(float("nan"))
        if dense:
            F.fgattn_dense_forward(self.q, self.k, self.v, p, self.out, self.lse, ws)
        else:
            F.fgattn_forward(self.q, self.k, self.v, self.d_indptr, self.d_indices, p, self.out, self.lse, ws)
        torch.cuda.synchronize()
        return out_to_f64(self.out), self.lse.double().cpu().numpy()


def gather_items(w, out, lse, items):
    """[B,H,L,d] / [B,H,L] -> per-item blocks [n, M, d] / [n, M] (NaN past L), matching the oracle's layout."""
    QB = w.QB
    o = out.reshape(-1, w.L, w.d)
    l = lse.reshape(-1, w.L)
    bo = np.full((len(items), w.M, w.d), np.nan)
    bl = np.full((len(items), w.M), np.nan)
    for n, it in enumerate(items):
        s, i = divmod(int(it), QB)
        r0, r1 = i * w.M, min((i + 1) * w.M, w.L)
        bo[n, :r1 - r0] = o[s, r0:r1]
        bl[n, :r1 - r0] = l[s, r0:r1]
    return bo, bl


def compare(got_out, got_lse, ref_out, ref_lse, what=""):
    """Asserts the benchmark's tolerances on rows the oracle defined (non-NaN); returns the error figures."""
    valid = ~np.isnan(ref_lse)
    assert not np.isnan(got_lse[valid]).any(), what + ": NaN lse in a defined row"
    assert not np.isnan(got_out[valid]).any(), what + ": NaN out in a defined row"
    eo = np.abs(got_out[valid] - ref_out[valid])
    fin = np.isfinite(ref_lse[valid])
    assert (got_lse[valid][~fin] == ref_lse[valid][~fin]).all(), what + ": -inf lse mismatch"
    el = np.abs(got_lse[valid][fin] - ref_lse[valid][fin]) / np.maximum(1.0, np.abs(ref_lse[valid][fin]))
    res = dict(max_abs=float(eo.max()) if eo.size else 0.0, mean_abs=float(eo.mean()) if eo.size else 0.0,
               lse_rel=float(el.max()) if el.size else 0.0)
    say("    %s: out max-abs %.3e mean-abs %.3e, lse rel %.3e" % (what, res["max_abs"], res["mean_abs"], res["lse_rel"]))
    assert res["max_abs"] <= OUT_MAX_ABS and res["mean_abs"] <= OUT_MEAN_ABS and res["lse_rel"] <= LSE_REL, what
    return res


def check_against_oracle(oracle, prob, got, items=None, what="", scale=None):
    w = prob.w
    if items is None:
        items = np.arange(w.items, dtype=np.int64)
    # (the C ABI takes scale as a float: the oracle gets the same number, not the double it was rounded from)
    ref_out, ref_lse = oracle.attention(prob.q_bits, prob.k_bits, prob.v_bits, w.M, w.N,
                                        float(np.float32(w.scale if scale is None else scale)), prob.indptr, prob.indices,
                                        items=items)
    bo, bl = gather_items(w, got[0], got[1], items)
    # rows past L must not have been written: the NaN poison is still there
    assert np.isnan(bl[np.isnan(ref_lse)]).all(), what + ": wrote a row past L"
    return compare(bo, bl, ref_out, ref_lse, what)


def sample_items(w, indptr, n_random, seed=0):
    """First block, last (partial) block, max- and min-length items, one item per head, plus random ones."""
    nnz = np.diff(indptr)
    rng = np.random.default_rng(seed)
    picks = {0, w.items - 1, w.QB - 1, int(np.argmax(nnz)), int(np.argmin(nnz))}
    for s in range(w.B * w.H):
        picks.add(s * w.QB + int(rng.integers(w.QB)))
    picks.update(int(x) for x in rng.integers(0, w.items, size=n_random))
    return np.array(sorted(picks), dtype=np.int64)
