#!/usr/bin/env python3
"""Times the forward kernel and the same build's dense kernel on the five benchmark configurations
(tiny, Wan-1.3B-shaped, the (M, N) sweep, HunyuanVideo-shaped, Wan-14B-shaped with per-head skew).
Prints one JSON object per line.

    python -m paper_2509_16518_amd.config_table [--steps 10] [--skip-hunyuan]
"""
import argparse
import json
import sys

import numpy as np

MFMA_BF16_PEAK_TFLOPS = 2500.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--skip-hunyuan", action="store_true")
    args = ap.parse_args()

    import torch
    from . import fgattn as F
    from . import workloads as W
    F.lib()
    if not torch.cuda.is_available():
        print("no GPU visible", file=sys.stderr)
        sys.exit(2)
    from .build import source_id
    print(json.dumps(dict(source_id(), script="paper_2509_16518_amd.config_table", argv=sys.argv[1:])), flush=True)

    def dev(bits):
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)

    def time_calls(fn, warmup, steps):
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

    configs = [("1 tiny", W.TINY), ("2 wan-1.3b", W.WAN_1_3B)]
    for M in (16, 64, 128):
        for N in (1, 8, 32, 64):
            configs.append(("3 sweep M=%d N=%d window" % (M, N), W.sweep(M, N)))
            configs.append(("3 sweep M=%d N=%d random" % (M, N), W.sweep(M, N, W.MASK_RANDOM)))
    if not args.skip_hunyuan:
        configs.append(("4 hunyuan", W.HUNYUAN))
    configs.append(("5 wan-14b-skew", W.WAN_14B_SKEW))

    for label, w in configs:
        q, k, v = W.make_qkv(w)
        indptr, indices = W.make_mask(w)
        useful, dense_flop = W.useful_flop(w, indptr, indices), W.dense_flop(w)
        dq, dk, dv = dev(q), dev(k), dev(v)
        del q, k, v
        d_indptr, d_indices = torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda()
        out = torch.empty_like(dq)
        lse = torch.empty(dq.shape[:3], dtype=torch.float32, device="cuda")
        p = F.make_params(dq, dk, dv, out, w.M, w.N, w.scale)
        p_reuse = F.make_params(dq, dk, dv, out, w.M, w.N, w.scale, F.FLAG_REUSE_PLAN)
        ws = torch.empty(F.fgattn_workspace_bytes(p), dtype=torch.uint8, device="cuda")
        steps = args.steps if w.items > 1000 else 10 * args.steps
        ms = time_calls(lambda: F.fgattn_forward(dq, dk, dv, d_indptr, d_indices, p, out, lse, ws), 2, steps)
        ms_main = time_calls(lambda: F.fgattn_forward(dq, dk, dv, d_indptr, d_indices, p_reuse, out, lse, ws), 2, steps)
        ms_dense = time_calls(lambda: F.fgattn_dense_forward(dq, dk, dv, p, out, lse, ws), 1, max(2, steps // 4))
        print(json.dumps({
            "config": label, "H": w.H, "L": w.L, "d": w.d, "M": w.M, "N": w.N,
            "realised_sparsity": 1.0 - indices.size / float(w.items * w.G), "nnz": int(indices.size),
            "ms": ms, "main_kernel_ms": ms_main, "useful_tflops": useful / ms / 1e9,
            "pct_bf16_mfma_peak": 100.0 * useful / ms / 1e9 / MFMA_BF16_PEAK_TFLOPS,
            "dense_equiv_tflops": dense_flop / ms / 1e9,
            "gather_request_GBps": indices.size * w.N * 4.0 * w.d / ms / 1e6,
            "dense_ms": ms_dense, "dense_tflops": dense_flop / ms_dense / 1e9, "sparse_over_dense": ms / ms_dense}), flush=True)
        del dq, dk, dv, out, lse, d_indptr, d_indices, ws
        torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
