#!/usr/bin/env python3
"""Benchmark of the FG-Attn forward hot path on one MI355X.

A "step" is one fgattn_forward call (ordering pre-pass + persistent sparse attention kernel)
on the Wan-2.1-1.3B-shaped synthetic workload (B=1, H=12, L=32760, d=128, M=64, N=1, 70%
sparsity: locality window on the 21x30x52 token grid plus seeded random fill), inputs
resident in HBM.  Prints ONE JSON line:
  value       useful (unskipped) TFLOP/s of the whole step
  roofline    the persistent forward kernel alone against the bf16 MFMA peak
  cpu_baseline  the fp64 oracle timed on the host cores on a sample of work items
  configs     the same kernel figures for the HunyuanVideo-shaped and the Wan-14B-shaped (skewed) workloads
plus the same build's dense kernel at 0% sparsity and the sparse/dense time ratio.
"""
import argparse
import json
import os
import re
import subprocess
import sys
import time

import numpy as np

REPO = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, REPO)

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def profiled_traffic(workload):
    """HBM bytes per launch of the forward kernel from the committed rocprofv3 summary of this workload (FETCH_SIZE /
    WRITE_SIZE runs scaled by the copy-kernel factors stated there).  The summary carries one machine-readable line
      <!-- bench: hbm_traffic_bytes_per_launch=<float> kernel_ms=<float> -->
    so that the figure is never typed in here; returns (bytes or None, source text)."""
    path = os.path.join(REPO, "profiles", "fgattn_fwd_kernel_%s.md" % workload)
    if not os.path.exists(path):
        return None, None
    m = re.search(r"<!--\s*bench:\s*hbm_traffic_bytes_per_launch=([0-9.eE+-]+)\s+kernel_ms=([0-9.eE+-]+)\s*-->", open(path).read())
    if not m:
        return None, None
    try:
        rev = subprocess.run(["git", "log", "-1", "--format=%h", "--", path], cwd=REPO, stdout=subprocess.PIPE,
                             stderr=subprocess.DEVNULL, text=True, timeout=10).stdout.strip()
    except Exception:
        rev = ""
    src = "profiles/%s%s, measured at kernel_ms=%s (not in this run)" % (os.path.basename(path), " @" + rev if rev else "", m.group(2))
    return float(m.group(1)), src


def time_calls(fn, warmup, steps):
    """HIP events on torch's current stream (the stream fn launches on), one pair around the timed region and one
    event between steps.  Returns dict(mean, median, min) in milliseconds per call."""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    ev[0].record()
    for i in range(steps):
        fn()
        ev[i + 1].record()
    torch.cuda.synchronize()
    each = np.array([ev[i].elapsed_time(ev[i + 1]) for i in range(steps)])
    return {"mean": ev[0].elapsed_time(ev[steps]) / steps, "median": float(np.median(each)), "min": float(each.min())}


def cpu_baseline(w, q, k, v, indptr, indices, n_items):
    """The oracle as it stands on a bounded sample of work items; returns the JSON object."""
    import oracle
    from paper_2509_16518_amd import workloads as W
    rng = np.random.default_rng(0)
    items = np.sort(rng.choice(w.items, size=n_items, replace=False)).astype(np.int64)
    keys = W.active_keys_per_item(w, indptr, indices)[items]
    rows = np.minimum(w.M, w.L - (items % w.QB) * w.M)
    flop = float(np.sum(rows * keys) * 4.0 * w.d)
    t0 = time.perf_counter()
    oracle.attention(q, k, v, w.M, w.N, w.scale, indptr, indices, items=items)
    dt = time.perf_counter() - t0
    return {"value": flop / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": "%d of %d work items (seeded random), %.1f s wall, fp64" % (n_items, w.items, dt),
            "extrapolated_full_s": dt * (W.useful_flop(w, indptr, indices) / flop)}


class Resident:
    """One workload uploaded to the GPU, with the closures the timings call."""

    def __init__(self, w):
        import torch
        from paper_2509_16518_amd import fgattn as F
        from paper_2509_16518_amd import workloads as W
        self.w = w
        log("generating %s inputs on the host" % w.name)
        self.q, self.k, self.v = W.make_qkv(w)
        self.indptr, self.indices = W.make_mask(w)
        self.useful = W.useful_flop(w, self.indptr, self.indices)
        self.dense_flop = W.dense_flop(w)
        self.density = self.indices.size / float(w.items * w.G)

        def dev(bits):
            return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
        self.dev = dev
        self.dq, self.dk, self.dv = dev(self.q), dev(self.k), dev(self.v)
        self.d_indptr, self.d_indices = torch.from_numpy(self.indptr).cuda(), torch.from_numpy(self.indices).cuda()
        self.out = torch.empty_like(self.dq)
        self.lse = torch.empty(self.dq.shape[:3], dtype=torch.float32, device="cuda")
        self.p = F.make_params(self.dq, self.dk, self.dv, self.out, w.M, w.N, w.scale)
        self.ws = torch.empty(F.fgattn_workspace_bytes(self.p), dtype=torch.uint8, device="cuda")
        self.p_reuse = F.make_params(self.dq, self.dk, self.dv, self.out, w.M, w.N, w.scale, F.FLAG_REUSE_PLAN)
        self.F = F

    def step(self):
        self.F.fgattn_forward(self.dq, self.dk, self.dv, self.d_indptr, self.d_indices, self.p, self.out, self.lse, self.ws)

    def kernel_only(self):   # plan already in the workspace
        self.F.fgattn_forward(self.dq, self.dk, self.dv, self.d_indptr, self.d_indices, self.p_reuse, self.out, self.lse,
                              self.ws)

    def dense(self, M):
        import torch
        F = self.F
        pd = F.make_params(self.dq, self.dk, self.dv, self.out, M, 1, self.w.scale)
        wsd = torch.empty(F.fgattn_workspace_bytes(pd), dtype=torch.uint8, device="cuda")
        return lambda: F.fgattn_dense_forward(self.dq, self.dk, self.dv, pd, self.out, self.lse, wsd)

    def describe(self):
        w = self.w
        return {"workload": "%s-shaped: B=%d H=%d L=%d d=%d M=%d N=%d, %s mask" %
                            (w.name, w.B, w.H, w.L, w.d, w.M, w.N,
                             "window+random-fill" if w.kind == 0 else "window+fill, per-head lognormal density"),
                "realised_sparsity": 1.0 - self.density, "nnz": int(self.indices.size), "work_items": int(w.items),
                "grid": self.F.fgattn_grid_size(self.p)}


def dense_figures(r, steps):
    """The same build's dense kernel at 0% sparsity, in both query tilings it has."""
    res = {}
    for M in sorted({r.w.M if r.w.M in (64, 128) else 128, 128}):
        t = time_calls(r.dense(M), 2, steps)
        res["%d_row_tiles" % M] = {"ms": t["mean"], "ms_median": t["median"], "tflops": r.dense_flop / t["mean"] / 1e9,
                                   "pct_bf16_mfma_peak": 100.0 * r.dense_flop / t["mean"] / 1e9 / MFMA_BF16_PEAK_TFLOPS,
                                   "steps": steps}
    return res


def extra_config(w, steps):
    """Kernel time, useful TFLOP/s, fraction of peak and the dense comparison for one more workload."""
    import torch
    r = Resident(w)
    ts = time_calls(r.step, 2, steps)
    tk = time_calls(r.kernel_only, 1, steps)
    res = {"config": r.describe(), "ms_per_step": ts["mean"], "ms_per_step_median": ts["median"],
           "kernel_ms": tk["mean"], "kernel_ms_median": tk["median"], "kernel_ms_min": tk["min"],
           "useful_tflops": r.useful / ts["mean"] / 1e9,
           "frac_bf16_mfma_peak_kernel": r.useful / tk["mean"] / 1e9 / MFMA_BF16_PEAK_TFLOPS,
           "dense_equiv_tflops": r.dense_flop / ts["mean"] / 1e9,
           "gather_request_GBps": r.indices.size * w.N * 4.0 * w.d / ts["mean"] / 1e6, "steps": steps}
    dense = dense_figures(r, max(2, steps // 2))
    best = min(dense.values(), key=lambda d: d["ms"])
    res["dense"] = dense
    res["sparse_over_dense_time"] = ts["mean"] / dense["%d_row_tiles" % (w.M if w.M in (64, 128) else 128)]["ms"]
    res["sparse_over_fastest_dense_time"] = ts["mean"] / best["ms"]
    traffic, traffic_src = profiled_traffic(w.name)
    if traffic is not None:
        res["traffic"], res["traffic_source"] = traffic, traffic_src
    del r
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="wan-1.3b", choices=["wan-1.3b", "tiny", "hunyuan", "wan-14b-skew"])
    ap.add_argument("--cpu-items", type=int, default=3072, help="work items the oracle is timed on (0 = skip)")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-mask", dest="mask", action="store_false", help="skip timing the top-p mask kernels")
    ap.add_argument("--no-extra-configs", dest="extra", action="store_false",
                    help="skip the HunyuanVideo-shaped and Wan-14B-shaped workloads reported under 'configs'")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy kernel (reference for scaling rocprofv3 FETCH/WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (heads and query blocks are independent, "
              "so they would shard across GPUs with no exchange step). Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2509_16518_amd import fgattn as F
    from paper_2509_16518_amd import workloads as W
    F.lib()   # fail loudly if the HIP library is missing: there is no fallback path
    if not torch.cuda.is_available():
        print("no GPU visible", file=sys.stderr)
        sys.exit(2)

    named = {"wan-1.3b": W.WAN_1_3B, "tiny": W.TINY, "hunyuan": W.HUNYUAN, "wan-14b-skew": W.WAN_14B_SKEW}
    w = named[args.workload]
    r = Resident(w)
    useful, dense_flop, indices = r.useful, r.dense_flop, r.indices

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    log("timing %d steps after %d warm-up" % (args.steps, args.warmup))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    t_step = time_calls(r.step, args.warmup, args.steps)
    wall = time.perf_counter() - t0
    ms_step = t_step["mean"]
    t_main = time_calls(r.kernel_only, 2, args.steps)
    ms_main = t_main["mean"]
    traffic, traffic_src = profiled_traffic(w.name)
    res = {
        "metric": "sparse attn kernel time + useful TFLOP/s (% bf16 MFMA peak) at 70% sparsity",
        "value": useful / ms_step / 1e9,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": r.describe(),
        "kernel_ms": ms_step, "ms_per_step_median": t_step["median"],
        "pct_bf16_mfma_peak": 100.0 * useful / ms_step / 1e9 / MFMA_BF16_PEAK_TFLOPS,
        "dense_equiv_tflops": dense_flop / ms_step / 1e9,
        "gather_request_GBps": indices.size * w.N * 4.0 * w.d / ms_step / 1e6,
        "roofline": {"bound": "mfma", "achieved": useful / ms_main / 1e9, "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": useful / ms_main / 1e9 / MFMA_BF16_PEAK_TFLOPS,
                     "traffic": traffic, "traffic_source": traffic_src,
                     "kernel": "fgattn_fwd_kernel", "kernel_ms": ms_main, "kernel_ms_median": t_main["median"],
                     "kernel_ms_min": t_main["min"],
                     "frac_at_median": useful / t_main["median"] / 1e9 / MFMA_BF16_PEAK_TFLOPS},
        "wall_s_timed_region": wall,
    }
    if w.M in (64, 128) and w.d == 128 and w.N == 1:
        # the two halves of the forward kernel timed apart on the same launch shape (results discarded)
        scratch_out = torch.empty_like(r.dq)
        scratch_lse = torch.empty_like(r.lse)

        def part(which):
            return lambda: F.fgattn_forward_part(r.dq, r.dk, r.dv, r.d_indptr, r.d_indices, r.p_reuse, scratch_out,
                                                 scratch_lse, r.ws, which)
        ms_gather = time_calls(part(F.PART_GATHER), 2, max(3, args.steps // 2))["mean"]
        ms_compute = time_calls(part(F.PART_COMPUTE), 2, max(3, args.steps // 2))["mean"]
        gather_bytes = indices.size * w.N * 4.0 * w.d
        res["parts"] = {"gather_only_ms": ms_gather, "compute_only_ms": ms_compute,
                        "gather_only_TBps": gather_bytes / ms_gather / 1e9,
                        "gather_TBps_in_full_kernel": gather_bytes / ms_main / 1e9,
                        "compute_only_pct_bf16_mfma_peak": 100.0 * useful / ms_compute / 1e9 / MFMA_BF16_PEAK_TFLOPS}
        if w.M == 64:
            # how the gather half alone responds to more rows in flight and to fewer issuing waves: the fraction of
            # the MFMA peak that the kernel could reach if everything else hid under its gathers
            ms_ring3 = time_calls(part(F.PART_GATHER_RING3), 2, max(3, args.steps // 2))["mean"]
            ms_one = time_calls(part(F.PART_GATHER_ONE_WG), 2, max(3, args.steps // 2))["mean"]
            cus = torch.cuda.get_device_properties(0).multi_processor_count
            clk = 2.4e9

            def per_cu(ms):
                return gather_bytes / (ms * 1e-3) / cus / clk
            res["parts"].update({
                "gather_only_k_ring_of_3_tiles_ms": ms_ring3, "gather_only_one_wg_per_cu_ms": ms_one,
                "gather_bytes_per_clk_per_cu_at_2.4GHz": {"8_waves_2_tile_rings": per_cu(ms_gather),
                                                          "8_waves_3_tile_k_ring": per_cu(ms_ring3),
                                                          "4_waves_2_tile_rings": per_cu(ms_one)},
                "frac_bf16_mfma_peak_if_gather_bound": {"2_tile_rings": useful / ms_gather / 1e9 / MFMA_BF16_PEAK_TFLOPS,
                                                        "3_tile_k_ring": useful / ms_ring3 / 1e9 / MFMA_BF16_PEAK_TFLOPS}})
        # the instruction-issue ceiling of the compute half: the same mix of MFMAs, exponentials and other vector
        # instructions per wave-tile as this tile shape's key loop, on the same occupancy, without memory traffic or barriers
        other = 67 if w.M == 64 else 61
        probe_scratch = torch.empty(2048 * torch.cuda.get_device_properties(0).multi_processor_count, dtype=torch.uint8, device="cuda")
        probe_flop = F.fgattn_issue_probe(other, 4000, probe_scratch)
        ms_mix = time_calls(lambda: F.fgattn_issue_probe(other, 4000, probe_scratch), 3, 10)["median"]
        ms_mfma = time_calls(lambda: F.fgattn_issue_probe(0, 4000, probe_scratch), 3, 10)["median"]
        res["parts"]["issue_ceiling"] = {
            "mix_per_wave_tile": "16 MFMA + 16 v_exp + %d other vector instructions" % other,
            "tflops_mfma_only": probe_flop / ms_mfma / 1e9, "tflops_at_this_mix": probe_flop / ms_mix / 1e9,
            "compute_only_over_ceiling": (useful / ms_compute) / (probe_flop / ms_mix)}
        del scratch_out, scratch_lse, probe_scratch
    if args.mask and w.grid[0] * w.grid[1] * w.grid[2] == w.L and w.name == "wan-1.3b":
        # the step before the hot path (Sec. 4.3): top-p mask from block means, on Q/K with space-time locality
        log("timing the top-p mask kernels")
        mq, mk = W.make_qk_local(w, gain=2.5)
        dmq, dmk = r.dev(mq), r.dev(mk)
        pm = F.make_params(dmq, dmk, dmk, dmq, w.M, w.N, w.scale)
        mws = torch.empty(F.fgattn_mask_workspace_bytes(pm), dtype=torch.uint8, device="cuda")
        m_indptr = torch.zeros(w.items + 1, dtype=torch.int64, device="cuda")
        ms_select = time_calls(lambda: F.fgattn_mask_select(dmq, dmk, pm, 0.9, m_indptr, mws), 2, 5)["mean"]
        m_nnz = int(m_indptr[-1].item())
        m_indices = torch.empty(m_nnz, dtype=torch.int32, device="cuda")
        ms_emit = time_calls(lambda: F.fgattn_mask_emit(pm, m_indptr, m_indices, mws), 2, 5)["mean"]
        res["mask"] = {"top_p": 0.9, "select_ms": ms_select, "emit_ms": ms_emit, "density": m_nnz / float(w.items * w.G),
                       "workspace_MB": mws.numel() / 1e6,
                       # scores written once and read once (the row of a query block then stays in LDS), one bit
                       # per score written and read, the ids written, Q and K read
                       "algorithmic_GB": (2 * w.items * w.G * 4.0 + 2 * w.items * w.G / 8.0 + 4.0 * m_nnz +
                                          2.0 * w.H * w.L * w.d * 2) / 1e9,
                       "data": "N(0,1) + random Fourier features of the token grid position (gain 2.5)"}
        del dmq, dmk, mws, m_indices
    if not args.no_dense:
        dense = dense_figures(r, max(3, args.steps // 4))
        own = dense["%d_row_tiles" % (w.M if w.M in (64, 128) else 128)]
        best = min(dense.values(), key=lambda d: d["ms"])
        res["dense"] = dict(own)
        res["sparse_over_dense_time"] = ms_step / own["ms"]
        res["dense_fastest_tiling"] = dict(best, sparse_over_dense_time=ms_step / best["ms"],
                                           tiling=min(dense, key=lambda kk: dense[kk]["ms"]))
        if "mask" in res:
            res["mask"]["over_dense_time"] = (res["mask"]["select_ms"] + res["mask"]["emit_ms"]) / own["ms"]
            res["mask"]["over_fastest_dense_time"] = (res["mask"]["select_ms"] + res["mask"]["emit_ms"]) / best["ms"]
    if args.cpu_items > 0:
        log("timing the oracle on %d work items" % args.cpu_items)
        res["cpu_baseline"] = cpu_baseline(w, r.q, r.k, r.v, r.indptr, r.indices, min(args.cpu_items, w.items))
    if args.extra and w.name == "wan-1.3b":
        del r
        torch.cuda.empty_cache()
        res["configs"] = {}
        for name in ("wan-14b-skew", "hunyuan"):
            log("extra config %s" % name)
            res["configs"][name] = extra_config(named[name], 5)
    from paper_2509_16518_amd.build import source_id
    res["source"] = source_id()
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
