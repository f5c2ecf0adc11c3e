#!/usr/bin/env python3
"""Sparsity sweep at a fixed square shape (the fifth benchmark configuration): for every
(V, M, C) point time venom_spmm and a dense fp16 GEMM of the same R x K x C on the same GPU and
print a markdown table (useful TFLOP/s, speedup over dense, ideal speedup M/2).

    python -m paper_2310_02065_amd.sweep [--V 128] [--C 2048] [--M 4 8 16 32 64 128] [--iters 60]
    python -m paper_2310_02065_amd.sweep --R 1024 --K 1024 4096 16384 --C 4096 --M 8 16 32   (a weight layer, varying K)
"""
from __future__ import annotations

import argparse
import sys


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--V", type=int, nargs="+", default=[128])
    ap.add_argument("--C", type=int, nargs="+", default=[2048])
    ap.add_argument("--M", type=int, nargs="+", default=[4, 8, 16, 32, 64, 128])
    ap.add_argument("--R", type=int, default=None, help="rows of A (default: the sweep shape, 8192)")
    ap.add_argument("--K", type=int, nargs="+", default=None, help="inner sizes (default: the sweep shape, 8192)")
    ap.add_argument("--iters", type=int, default=60)
    args = ap.parse_args()

    import numpy as np
    import torch
    from . import binding, inputs

    if not torch.cuda.is_available():
        print("no GPU visible", file=sys.stderr)
        sys.exit(3)
    binding.lib()
    dev = torch.device("cuda:0")
    R = args.R or inputs.SWEEP_SHAPE[0]
    Ks = args.K or [inputs.SWEEP_SHAPE[1]]

    def timed(fn, iters):
        for _ in range(10):
            fn()
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
        for a, b in ev:
            a.record(); fn(); b.record()
        torch.cuda.synchronize()
        t = sorted(a.elapsed_time(b) for a, b in ev)
        return t[len(t) // 2]

    print("| R x K | V | M | C | spmm ms | useful TFLOP/s | dense GEMM ms | speedup | ideal |")
    print("|---|---|---|---|---|---|---|---|---|")
    for K, C in [(K, C) for K in Ks for C in args.C]:
        dense_ms = None
        for V in args.V:
            for M in args.M:
                A_bits, mask, B_bits = inputs.gen_problem(R, K, C, V, M, 1.0, seed=inputs.config_seed(4) + 7 * M + V + C)
                A_d = torch.from_numpy(A_bits.view(np.float16)).to(dev)
                B_d = torch.from_numpy(B_bits.view(np.float16)).to(dev)
                h = binding.venom_compress(A_d, torch.from_numpy(mask).to(dev), V, 2, M)
                out = torch.empty((R, C), dtype=torch.float16, device=dev)
                ms = timed(lambda: binding.venom_spmm(h, B_d, out=out), args.iters)
                if dense_ms is None:
                    D = torch.empty((R, C), dtype=torch.float16, device=dev)
                    dense_ms = timed(lambda: torch.matmul(A_d, B_d, out=D), max(10, args.iters // 3))
                    del D
                useful = 2.0 * R * C * K * 2 / M
                print(f"| {R} x {K} | {V} | {M} | {C} | {ms:.4f} | {useful / ms * 1e-9:.0f} | {dense_ms:.4f} | {dense_ms / ms:.2f} | {M / 2:.0f} |",
                      flush=True)
                h.close()
                del A_d, B_d, out, h


if __name__ == "__main__":
    main()
