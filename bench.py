#!/usr/bin/env python3
"""Benchmark of the V:N:M sparse x dense product on one MI355X.

A "step" is one pass of the whole hot path -- one venom_spmm launch (column-loc fetch, gathered B
loads, values + metadata stream, 2:4 matrix instructions, output stage) -- over one synthetic
workload whose operands are already resident in HBM.  The headline workload is the GPT-3-175B
FFN-up shape (A 49152 x 12288 in 128:2:32, B 12288 x 2048), the one the 50 %-of-MFMA-peak target
is stated on.  Prints ONE JSON line:

  metric/value     useful TFLOP/s = 2*R*C*K*N/M / t  (N/M of the dense operation count)
  roofline         the product kernel against the dense fp16 MFMA peak (the 2:4 instruction
                   performs useful FLOPs at exactly the dense instruction's FLOP rate), with the
                   kernel's average duration measured by HIP events on its own stream
  dense_gemm       torch.matmul (hipBLASLt) of the same R x K x C on the same GPU, same loop
  cpu_baseline     the fp64 oracle (expand + dgemm) timed on the host cores on a row sample
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP16_MFMA_TFLOPS = 2500.0     # MI355X dense fp16 matrix peak
PEAK_HBM_GBS = 8000.0

# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (see profiles/),
# scaled by the same counters read on a plain copy kernel; None where not measured yet.
MEASURED_TRAFFIC_BYTES = {
    "gpt3": 1125849804,                    # 924.5 MB read + 201.3 MB written
    "bert_large": 187424768,               # 53.2 MB read + 134.2 MB written
    "sweep_v128_m128_c2048": 86499328,     # 52.9 MB read + 33.6 MB written
    "sweep_v128_m32_c256": 36153344,       # 32.0 MB read + 4.2 MB written
}


def algorithmic_bytes(R, K, C, V, M, out_bytes=2):
    """Bytes the method has to move from/to HBM once: values, metadata, column-loc, B, C."""
    G = K // M
    return 2 * R * G * 2 + R * G // 2 + (R // V) * G * 4 * 2 + 2 * K * C + out_bytes * R * C


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="gpt3", help="gpt3 | bert_large | bert_base | tiny | sweep_v{V}_m{M}_c{C}")
    ap.add_argument("--variant", type=int, default=-1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch three plain 1 GiB device copies (for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives or sharding are part of it); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2310_02065_amd import binding, inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    binding.lib()   # fail loudly if the HIP library is missing
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    names = list(inputs.CONFIGS)
    if args.workload in inputs.CONFIGS:
        R, K, C, V, M, sigma = inputs.CONFIGS[args.workload]
        seed = inputs.config_seed(names.index(args.workload))
    else:
        # a point of the sparsity sweep: "sweep_v{V}_m{M}_c{C}", e.g. sweep_v128_m32_c256 (bandwidth-bound)
        parts = dict((p[0], int(p[1:])) for p in args.workload.split("_")[1:])
        V, M, C = parts["v"], parts["m"], parts["c"]
        R, K = inputs.SWEEP_SHAPE
        sigma = 1.0
        seed = inputs.config_seed(4) + 7 * M + V + C
    N = 2
    t0 = time.time()
    A_bits, mask, B_bits = inputs.gen_problem(R, K, C, V, M, sigma, seed=seed)
    t_gen = time.time() - t0

    A_d = torch.from_numpy(A_bits.view(np.float16)).to(dev)
    mask_d = torch.from_numpy(mask).to(dev)
    B_d = torch.from_numpy(B_bits.view(np.float16)).to(dev)
    h = binding.venom_compress(A_d, mask_d, V, N, M)
    dense_A = None
    if not args.no_dense:
        dense_A = binding.venom_decompress(h)     # the expanded masked matrix for the dense comparator
    del A_d, mask_d
    C_d = torch.empty((R, C), dtype=torch.float16, device=dev)

    def timed(fn, steps, warmup):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        t_start = time.perf_counter()
        for a, b in evs:
            a.record()
            fn()
            b.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t_start) * 1e3
        per = sorted(a.elapsed_time(b) for a, b in evs)
        return wall_ms / steps, sum(per) / len(per), per[len(per) // 2], per[0]

    step = lambda: binding.venom_spmm(h, B_d, out=C_d, variant=args.variant)
    ms_wall, ms_avg, ms_med, ms_min = timed(step, args.steps, args.warmup)

    useful_flop = 2.0 * R * C * K * N / M
    dense_flop = 2.0 * R * C * K
    value = useful_flop / (ms_wall * 1e-3) / 1e12
    kern_tflops = useful_flop / (ms_avg * 1e-3) / 1e12

    alg_bytes = algorithmic_bytes(R, K, C, V, M)
    t_mfma = useful_flop / (PEAK_FP16_MFMA_TFLOPS * 1e12)
    t_hbm = alg_bytes / (PEAK_HBM_GBS * 1e9)
    if t_mfma >= t_hbm:
        roofline = {"bound": "mfma", "achieved": round(kern_tflops, 2), "peak": PEAK_FP16_MFMA_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(kern_tflops / PEAK_FP16_MFMA_TFLOPS, 4)}
    else:
        gbs = alg_bytes / (ms_avg * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": round(gbs / PEAK_HBM_GBS, 4)}
    roofline["traffic"] = MEASURED_TRAFFIC_BYTES.get(args.workload)
    roofline["kernel_ms_avg"] = round(ms_avg, 5)
    roofline["algorithmic_bytes"] = alg_bytes
    roofline["useful_flop"] = useful_flop

    out = {
        "metric": "V:N:M SpMM useful TFLOP/s (fp16)", "value": round(value, 2), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_wall, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: A {R}x{K} fp16 in {V}:{N}:{M}, B {K}x{C} fp16, C fp16 (fp32 accumulate)",
                   "R": R, "K": K, "C": C, "V": V, "N": N, "M": M, "seed": seed,
                   "variant": binding.venom_spmm_variants()[args.variant] if args.variant >= 0 else "auto"},
        "dense_equivalent_tflops": round(dense_flop / (ms_wall * 1e-3) / 1e12, 2),
        "frac_of_fp16_mfma_peak_useful": round(value / PEAK_FP16_MFMA_TFLOPS, 4),
        "kernel_ms": {"avg": round(ms_avg, 5), "median": round(ms_med, 5), "min": round(ms_min, 5)},
        "roofline": roofline,
    }

    if dense_A is not None:
        D_d = torch.empty((R, C), dtype=torch.float16, device=dev)
        dense = lambda: torch.matmul(dense_A, B_d, out=D_d)
        d_wall, d_avg, d_med, d_min = timed(dense, max(5, args.steps // 5), max(2, args.warmup // 5))
        out["dense_gemm"] = {"ms": round(d_avg, 5), "tflops": round(dense_flop / (d_avg * 1e-3) / 1e12, 2),
                             "speedup_of_spmm": round(d_avg / ms_avg, 3), "ideal_speedup": M / N,
                             "kind": "torch.matmul fp16 (hipBLASLt), same R x K x C, expanded masked A"}
        del D_d, dense_A

    if not args.no_cpu_baseline:
        from oracle import vnm_oracle as o
        v_d, c_d, m_d = binding.venom_export(h)
        torch.cuda.synchronize()
        v = v_d.cpu().numpy().view(np.uint16)
        c = c_d.cpu().numpy().view(np.uint16)
        m = m_d.cpu().numpy().view(np.uint32)
        cores = len(os.sched_getaffinity(0))

        def run_rows(nrows):
            t = time.perf_counter()
            o.spmm_fp64(v[:nrows], c[:nrows // V], m[:nrows], nrows, K, V, M, B_bits)
            return time.perf_counter() - t

        probe_rows = min(R, max(V, (2048 // V) * V))
        t_probe = run_rows(probe_rows)
        rows = int(min(R, max(probe_rows, (args.cpu_seconds / max(t_probe, 1e-6)) * probe_rows)))
        rows = max(V, rows // V * V)
        t_cpu = run_rows(rows) if rows != probe_rows else t_probe
        cpu_useful = 2.0 * rows * C * K * N / M
        out["cpu_baseline"] = {"value": round(cpu_useful / t_cpu / 1e12, 6), "unit": "TFLOP/s", "cores": cores,
                               "kind": "oracle",
                               "sample": f"first {rows} of {R} rows of the same workload (expand to dense + fp64 "
                                         f"matmul for C* and the bound matrix), {t_cpu:.2f} s"}
    if args.copy_calibration:
        # a plain copy kernel of known size: 2^30 bytes read, 2^30 bytes written per launch
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        out["copy_calibration"] = {"bytes_read": 1 << 30, "bytes_written": 1 << 30, "launches": 3}
        del src, dst
    out["host_seconds"] = {"generate_inputs": round(t_gen, 1)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
