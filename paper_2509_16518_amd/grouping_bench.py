#!/usr/bin/env python3
"""Grouped vs ungrouped query tiles (paper Sec. 4.2 / Sec. 5.1 "at different sparsities").

For query-tile sizes below 128 the paper merges R = 128/M tiles into one thread block, either consecutive tiles
or tiles with similar key sets (greedy merge-XOR), and reports planning and kernel time apart.  This script times,
on the same masks: the ungrouped kernel (this library runs small tiles natively), and the grouped kernel with both
groupings, with the grouping pre-pass ("planning") timed separately.  Prints one JSON object per line.

    python -m paper_2509_16518_amd.grouping_bench [--heads 12] [--tokens 32760] [--steps 5] [--density 0.3]
"""
import argparse
import json
import sys

import numpy as np


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--heads", type=int, default=12)
    ap.add_argument("--tokens", type=int, default=32760)
    ap.add_argument("--grid", type=int, nargs=3, default=[21, 30, 52])
    ap.add_argument("--head-dim", type=int, default=128)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--blocks", type=int, nargs="*", default=[64, 32, 16])
    ap.add_argument("--density", type=float, default=0.30, help="1 - sparsity of the masks (the paper uses 0.3 and 0.5)")
    args = ap.parse_args()

    import torch
    from . import fgattn as F
    from . import workloads as W
    F.lib()
    if not torch.cuda.is_available():
        print("no GPU visible", file=sys.stderr)
        sys.exit(2)
    from .build import source_id
    print(json.dumps(dict(source_id(), script="paper_2509_16518_amd.grouping_bench", argv=sys.argv[1:])), flush=True)

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

    base = W.Workload("grouping-bench", H=args.heads, L=args.tokens, d=args.head_dim, M=128, N=128, seed=8000)
    q, k, v = W.make_qkv(base)
    dq, dk, dv = dev(q), dev(k), dev(v)
    out = torch.empty_like(dq)
    lse = torch.empty(dq.shape[:3], dtype=torch.float32, device="cuda")

    masks = [("random", W.MASK_RANDOM, (0, 0, 0)), ("window+fill", W.MASK_WINDOW_FILL, (2, 4, 4))]
    for blk in args.blocks:
        for mname, kind, window in masks:
            w = W.Workload(base.name, H=base.H, L=base.L, d=base.d, M=blk, N=blk, grid=tuple(args.grid), window=window,
                           kind=kind, density=args.density, seed=8000 + blk)
            indptr, indices = W.make_mask(w)
            useful = W.useful_flop(w, indptr, indices)
            d_indptr, d_indices = torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda()
            p = F.make_params(dq, dk, dv, out, w.M, w.N, w.scale)
            ws = torch.empty(F.fgattn_workspace_bytes(p), dtype=torch.uint8, device="cuda")
            ms_plain = time_calls(lambda: F.fgattn_forward(dq, dk, dv, d_indptr, d_indices, p, out, lse, ws), 2, args.steps)
            row = {"block": "%dx%d" % (blk, blk), "mask": mname, "density": indices.size / float(w.items * w.G),
                   "ungrouped_ms": ms_plain, "ungrouped_tflops": useful / ms_plain / 1e9}
            R = 128 // blk
            NG = (w.QB + R - 1) // R
            groups = w.B * w.H * NG
            for mode, mid in (("consecutive", F.GROUP_CONSECUTIVE), ("xor", F.GROUP_XOR)):
                gws = torch.empty(F.fgattn_group_workspace_bytes(p, mid), dtype=torch.uint8, device="cuda")
                tiles = torch.empty(groups * R, dtype=torch.int32, device="cuda")
                up = torch.empty(groups + 1, dtype=torch.int64, device="cuda")
                ms_sel = time_calls(lambda: F.fgattn_group_select(d_indptr, d_indices, p, mid, tiles, up, gws), 1, 3)
                nnz = int(up[-1].item())
                ui = torch.empty(nnz, dtype=torch.int32, device="cuda")
                um = torch.empty(nnz, dtype=torch.uint8, device="cuda")
                ms_emit = time_calls(lambda: F.fgattn_group_emit(p, mid, tiles, up, ui, um, gws), 1, 3)
                ms_g = time_calls(lambda: F.fgattn_forward_grouped(dq, dk, dv, tiles, up, ui, um, p, out, lse, ws), 2,
                                  args.steps)
                row[mode] = {"plan_ms": ms_sel + ms_emit, "kernel_ms": ms_g, "useful_tflops": useful / ms_g / 1e9,
                             "union_density": nnz / float(groups * w.G),
                             "key_blocks_loaded_vs_ungrouped": nnz / float(indices.size)}
                del gws, ui, um
            print(json.dumps(row), flush=True)


if __name__ == "__main__":
    main()
