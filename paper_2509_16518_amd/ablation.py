#!/usr/bin/env python3
"""Skew x sparsity ablation of the forward kernel (paper Sec. 5.1, "at different levels of skew, sparsity").

For each (sparsity, skew) a mask is drawn with the paper's generator -- per query block a list length uniform in
[(1 - skew) * Lmax, Lmax] and that many random key blocks, Lmax chosen so that the mean density is the target --
at block size 128 x 32 (or --block-m / --block-n), and the sparse kernel is timed with the longest-first work queue and with static
assignment of query blocks to workgroups (the paper's "no scheduler"), next to the same build's dense kernel.
Prints one JSON object per line.

    python -m paper_2509_16518_amd.ablation [--heads 12] [--tokens 32760] [--steps 10] [--block-m 128 --block-n 32]
"""
import argparse
import json
import sys

import numpy as np


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--heads", type=int, default=12)
    ap.add_argument("--tokens", type=int, default=32760)
    ap.add_argument("--head-dim", type=int, default=128)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--block-m", type=int, default=128, help="query rows per block")
    ap.add_argument("--block-n", type=int, default=32, help="keys per block")
    ap.add_argument("--sparsity", type=float, nargs="*", default=[0.5, 0.7, 0.9])
    ap.add_argument("--skew", type=float, nargs="*", default=[0.0, 0.25, 0.5, 0.75, 1.0])
    args = ap.parse_args()

    import torch
    from . import fgattn as F
    from . import workloads as W
    F.lib()
    if not torch.cuda.is_available():
        print("no GPU visible", file=sys.stderr)
        sys.exit(2)
    from .build import source_id
    print(json.dumps(dict(source_id(), script="paper_2509_16518_amd.ablation", argv=sys.argv[1:])), flush=True)

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

    base = W.Workload("skew-ablation", H=args.heads, L=args.tokens, d=args.head_dim, M=args.block_m, N=args.block_n,
                      kind=W.MASK_SKEW_LEN, seed=7000)
    q, k, v = W.make_qkv(base)
    dq, dk, dv = dev(q), dev(k), dev(v)
    out = torch.empty_like(dq)
    lse = torch.empty(dq.shape[:3], dtype=torch.float32, device="cuda")
    p = F.make_params(dq, dk, dv, out, base.M, base.N, base.scale)
    p_static = F.make_params(dq, dk, dv, out, base.M, base.N, base.scale, F.FLAG_STATIC_ASSIGN)
    ws = torch.empty(F.fgattn_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    dense_ms = time_calls(lambda: F.fgattn_dense_forward(dq, dk, dv, p, out, lse, ws), 2, max(3, args.steps // 2))
    dense_flop = W.dense_flop(base)
    print(json.dumps({"kernel": "dense", "ms": dense_ms, "tflops": dense_flop / dense_ms / 1e9}), flush=True)

    for sparsity in args.sparsity:
        for skew in args.skew:
            w = W.Workload(base.name, H=base.H, L=base.L, d=base.d, M=base.M, N=base.N, kind=W.MASK_SKEW_LEN,
                           density=1.0 - sparsity, skew=skew, seed=7000 + int(1000 * sparsity) + int(100 * skew))
            indptr, indices = W.make_mask(w)
            lens = np.diff(indptr)
            useful = W.useful_flop(w, indptr, indices)
            d_indptr, d_indices = torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda()
            ms_q = time_calls(lambda: F.fgattn_forward(dq, dk, dv, d_indptr, d_indices, p, out, lse, ws), 2, args.steps)
            ms_s = time_calls(lambda: F.fgattn_forward(dq, dk, dv, d_indptr, d_indices, p_static, out, lse, ws), 2,
                              args.steps)
            print(json.dumps({
                "sparsity": sparsity, "skew": skew,
                "realised_sparsity": 1.0 - indices.size / float(w.items * w.G),
                "realised_skew": float(lens.max() - lens.min()) / float(lens.max()),
                "scheduler_ms": ms_q, "scheduler_tflops": useful / ms_q / 1e9,
                "static_ms": ms_s, "static_tflops": useful / ms_s / 1e9,
                "scheduler_gain": ms_s / ms_q, "speedup_over_dense": dense_ms / ms_q}), flush=True)


if __name__ == "__main__":
    main()
