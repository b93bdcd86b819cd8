#!/usr/bin/env python3
"""Benchmark of the FG-Attn forward hot path on one MI355X.

A "step" is one fgattn_forward call (ordering pre-pass + persistent sparse attention kernel)
on the Wan-2.1-1.3B-shaped synthetic workload (B=1, H=12, L=32760, d=128, M=64, N=1, 70%
sparsity: locality window on the 21x30x52 token grid plus seeded random fill), inputs
resident in HBM.  Prints ONE JSON line:
  value       useful (unskipped) TFLOP/s of the whole step
  roofline    the persistent forward kernel alone against the bf16 MFMA peak
  cpu_baseline  the fp64 oracle timed on the host cores on a sample of work items
plus the same build's dense kernel at 0% sparsity and the sparse/dense time ratio.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

REPO = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, REPO)

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak
# HBM bytes per launch of the forward kernel on the wan-1.3b workload, from the FETCH_SIZE / WRITE_SIZE
# rocprofv3 runs summarised in profiles/fgattn_fwd_kernel_wan-1.3b.md (scaled by the copy-kernel factors there)
HBM_TRAFFIC_BYTES = {"wan-1.3b": 2.06e9}


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def time_calls(fn, warmup, steps):
    """Mean milliseconds per call, HIP events on torch's current stream (the stream fn launches on)."""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="wan-1.3b", choices=["wan-1.3b", "tiny"])
    ap.add_argument("--cpu-items", type=int, default=3072, help="work items the oracle is timed on (0 = skip)")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-mask", dest="mask", action="store_false", help="skip timing the top-p mask kernels")
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

    w = {"wan-1.3b": W.WAN_1_3B, "tiny": W.TINY}[args.workload]
    log("generating %s inputs on the host" % w.name)
    q, k, v = W.make_qkv(w)
    indptr, indices = W.make_mask(w)
    useful = W.useful_flop(w, indptr, indices)
    dense_flop = W.dense_flop(w)
    density = indices.size / float(w.items * w.G)

    def dev(bits):
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    dq, dk, dv = dev(q), dev(k), dev(v)
    d_indptr, d_indices = torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda()
    out = torch.empty_like(dq)
    lse = torch.empty(dq.shape[:3], dtype=torch.float32, device="cuda")
    p = F.make_params(dq, dk, dv, out, w.M, w.N, w.scale)
    ws = torch.empty(F.fgattn_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    p_reuse = F.make_params(dq, dk, dv, out, w.M, w.N, w.scale, F.FLAG_REUSE_PLAN)

    def step():
        F.fgattn_forward(dq, dk, dv, d_indptr, d_indices, p, out, lse, ws)

    def main_kernel_only():
        F.fgattn_forward(dq, dk, dv, d_indptr, d_indices, p_reuse, out, lse, ws)

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
    ms_step = time_calls(step, args.warmup, args.steps)
    wall = time.perf_counter() - t0
    ms_main = time_calls(main_kernel_only, 2, args.steps)   # plan already in the workspace
    res = {
        "metric": "sparse attn kernel time + useful TFLOP/s (% bf16 MFMA peak) at 70% sparsity",
        "value": useful / ms_step / 1e9,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s-shaped: B=%d H=%d L=%d d=%d M=%d N=%d, window+random-fill mask" %
                               (w.name, w.B, w.H, w.L, w.d, w.M, w.N),
                   "realised_sparsity": 1.0 - density, "nnz": int(indices.size), "work_items": int(w.items),
                   "grid": F.fgattn_grid_size(p)},
        "kernel_ms": ms_step,
        "pct_bf16_mfma_peak": 100.0 * useful / ms_step / 1e9 / MFMA_BF16_PEAK_TFLOPS,
        "dense_equiv_tflops": dense_flop / ms_step / 1e9,
        "gather_request_GBps": indices.size * w.N * 4.0 * w.d / ms_step / 1e6,
        "roofline": {"bound": "mfma", "achieved": useful / ms_main / 1e9, "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": useful / ms_main / 1e9 / MFMA_BF16_PEAK_TFLOPS,
                     "traffic": HBM_TRAFFIC_BYTES.get(w.name),
                     "kernel": "fgattn_fwd_kernel", "kernel_ms": ms_main},
        "wall_s_timed_region": wall,
    }
    if w.M == 64 and w.d == 128 and w.N == 1:
        # the two halves of the forward kernel timed apart on the same launch shape (results discarded)
        scratch_out = torch.empty_like(dq)
        scratch_lse = torch.empty_like(lse)

        def part(which):
            return lambda: F.fgattn_forward_part(dq, dk, dv, d_indptr, d_indices, p_reuse, scratch_out, scratch_lse,
                                                 ws, which)
        ms_gather = time_calls(part(F.PART_GATHER), 2, max(3, args.steps // 2))
        ms_compute = time_calls(part(F.PART_COMPUTE), 2, max(3, args.steps // 2))
        gather_bytes = indices.size * w.N * 4.0 * w.d
        res["parts"] = {"gather_only_ms": ms_gather, "compute_only_ms": ms_compute,
                        "gather_only_TBps": gather_bytes / ms_gather / 1e9,
                        "gather_TBps_in_full_kernel": gather_bytes / ms_main / 1e9,
                        "compute_only_pct_bf16_mfma_peak": 100.0 * useful / ms_compute / 1e9 / MFMA_BF16_PEAK_TFLOPS}
        del scratch_out, scratch_lse
    if args.mask and w.grid[0] * w.grid[1] * w.grid[2] == w.L:
        # the step before the hot path (Sec. 4.3): top-p mask from block means, on Q/K with space-time locality
        log("timing the top-p mask kernels")
        mq, mk = W.make_qk_local(w, gain=2.5)
        dmq, dmk = dev(mq), dev(mk)
        pm = F.make_params(dmq, dmk, dmk, dmq, w.M, w.N, w.scale)
        mws = torch.empty(F.fgattn_mask_workspace_bytes(pm), dtype=torch.uint8, device="cuda")
        m_indptr = torch.zeros(w.items + 1, dtype=torch.int64, device="cuda")
        ms_select = time_calls(lambda: F.fgattn_mask_select(dmq, dmk, pm, 0.9, m_indptr, mws), 2, 5)
        m_nnz = int(m_indptr[-1].item())
        m_indices = torch.empty(m_nnz, dtype=torch.int32, device="cuda")
        ms_emit = time_calls(lambda: F.fgattn_mask_emit(pm, m_indptr, m_indices, mws), 2, 5)
        res["mask"] = {"top_p": 0.9, "select_ms": ms_select, "emit_ms": ms_emit, "density": m_nnz / float(w.items * w.G),
                       "workspace_MB": mws.numel() / 1e6,
                       # scores written once and read once (the row of a query block then stays in LDS), one bit
                       # per score written and read, the ids written, Q and K read
                       "algorithmic_GB": (2 * w.items * w.G * 4.0 + 2 * w.items * w.G / 8.0 + 4.0 * m_nnz +
                                          2.0 * w.H * w.L * w.d * 2) / 1e9,
                       "data": "N(0,1) + random Fourier features of the token grid position (gain 2.5)"}
        del dmq, dmk, mws, m_indices
    if not args.no_dense:
        def dense_step():
            F.fgattn_dense_forward(dq, dk, dv, p, out, lse, ws)
        nd = max(3, args.steps // 4)
        ms_dense = time_calls(dense_step, 2, nd)
        res["dense"] = {"ms": ms_dense, "tflops": dense_flop / ms_dense / 1e9,
                        "pct_bf16_mfma_peak": 100.0 * dense_flop / ms_dense / 1e9 / MFMA_BF16_PEAK_TFLOPS, "steps": nd}
        res["sparse_over_dense_time"] = ms_step / ms_dense
        if w.M != 128:
            # the dense kernel does not depend on the mask's tile size: also time it with 128-row query tiles,
            # its fastest tiling, so that the sparse step is also compared with the best dense kernel of this build
            p128 = F.make_params(dq, dk, dv, out, 128, 1, w.scale)
            ws128 = torch.empty(F.fgattn_workspace_bytes(p128), dtype=torch.uint8, device="cuda")
            ms_d128 = time_calls(lambda: F.fgattn_dense_forward(dq, dk, dv, p128, out, lse, ws128), 2, nd)
            res["dense_128_row_tiles"] = {"ms": ms_d128, "tflops": dense_flop / ms_d128 / 1e9,
                                          "sparse_over_dense_time": ms_step / ms_d128}
        if "mask" in res:
            res["mask"]["over_dense_time"] = (res["mask"]["select_ms"] + res["mask"]["emit_ms"]) / ms_dense
    if args.cpu_items > 0:
        log("timing the oracle on %d work items" % args.cpu_items)
        res["cpu_baseline"] = cpu_baseline(w, q, k, v, indptr, indices, min(args.cpu_items, w.items))
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
