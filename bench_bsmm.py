#!/usr/bin/env python3
"""Throughput of the general block-sparse products (dmoe_bsmm) on a random 128x128 block mask: the six products
of Sections 4.2 / 5.1, and DDS, on a topology that is NOT block-diagonal.  One JSON line; flops = 2 * nnz * 128 * 128 * D.

    python bench_bsmm.py [--block-rows 64] [--block-cols 64] [--density 0.5] [--dense 1024] [--iters 20]
"""
from __future__ import annotations

import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--block-rows", type=int, default=64)
    ap.add_argument("--block-cols", type=int, default=64)
    ap.add_argument("--density", type=float, default=0.5)
    ap.add_argument("--dense", type=int, default=1024)
    ap.add_argument("--iters", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    args = ap.parse_args()

    import numpy as np
    import torch
    import paper_2211_15841_amd as dm
    assert torch.cuda.is_available(), "needs a GPU"
    torch.cuda.set_device(0)
    rng = np.random.default_rng(4242)
    mask = (rng.random((args.block_rows, args.block_cols)) < args.density).astype(np.uint8)
    bs = dm.BlockSparse(mask)
    M, N, D = args.block_rows * 128, args.block_cols * 128, args.dense
    g = torch.Generator(device="cuda").manual_seed(7)
    x = torch.randn(M, D, device="cuda", generator=g).to(torch.bfloat16)
    w_dn = (0.05 * torch.randn(D, N, device="cuda", generator=g)).to(torch.bfloat16)
    w_nd = (0.05 * torch.randn(N, D, device="cuda", generator=g)).to(torch.bfloat16)
    s = torch.randn(bs.nnz, 128, 128, device="cuda", generator=g).to(torch.bfloat16)
    xt = torch.randn(D, M, device="cuda", generator=g).to(torch.bfloat16)
    ops = {
        "sdd": lambda: bs.sdd(x, w_dn), "dsd": lambda: bs.dsd(s, w_nd), "sddt": lambda: bs.sddt(x, w_nd),
        "dstd": lambda: bs.dstd(s, x), "dsdt": lambda: bs.dsdt(s, w_dn), "ddts": lambda: bs.ddts(x, s),
        "dds": lambda: bs.dds(xt, s),
    }
    flops = 2.0 * bs.nnz * 128 * 128 * D
    out = {}
    for name, fn in ops.items():
        for _ in range(args.warmup):
            fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(args.iters):
            fn()
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / args.iters
        out[name] = {"ms": round(ms, 4), "tflops": round(flops / ms / 1e9, 1)}
        print("[bsmm] %-5s %.3f ms  %.0f TFLOP/s" % (name, ms, flops / ms / 1e9), file=sys.stderr, flush=True)
    tf = [v["tflops"] for v in out.values()]
    print(json.dumps({"metric": "general block-sparse products on a random block mask, TFLOP/s (bf16)",
                      "unit": "TFLOP/s", "mean": round(sum(tf) / len(tf), 1), "min": min(tf), "max": max(tf),
                      "config": {"block_rows": args.block_rows, "block_cols": args.block_cols,
                                 "density": args.density, "nnz_blocks": bs.nnz, "dense": D, "block": 128},
                      "dtype": "bf16", "data": "synthetic", "note": "includes one output allocation per call",
                      "products": out}))


if __name__ == "__main__":
    main()
