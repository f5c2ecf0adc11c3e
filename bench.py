#!/usr/bin/env python3
"""Benchmark of the V:N:M sparse x dense product on one MI355X.

A "step" is one pass of the whole hot path -- one venom_spmm launch (column-loc fetch, gathered B
loads, values + metadata stream, 2:4 matrix instructions, output stage) -- over one synthetic
workload whose operands are already resident in HBM.  The headline workload is the GPT-3-175B
FFN-up shape (A 49152 x 12288 in 128:2:32, B 12288 x 2048), the one the 50 %-of-MFMA-peak target
is stated on.  Prints ONE JSON line:

  metric/value     useful TFLOP/s = 2*R*C*K*N/M / t  (N/M of the dense operation count), wall-timed
  roofline         the product kernel against the dense fp16 MFMA peak (the 2:4 instruction
                   performs useful FLOPs at exactly the dense instruction's FLOP rate), with the
                   kernel's average duration measured by HIP events on its own stream
  dense_gemm       torch.matmul (hipBLASLt) of the same R x K x C on the same GPU, same loop
  measured_peak    the 2:4 matrix instruction alone (register operands), timed here: the rate the
                   GPU sustains at the clock it holds under that load
  hbm_calibration  plain fill / copy of 1 GiB on the same GPU: the HBM rates linear streams sustain
  cold_operands    the headline launches with the compressed matrix, B and C rotated through more
                   memory than the caches hold (weights of a deep model arrive from HBM, not from a cache)
  calls            the other entry points on the headline matrix: fused bias / GELU, the token-major
                   layer call, magnitude pruning, compression
  configs          the other workloads (tiny, BERT-base, BERT-large, the C = 2048 column of the
                   sparsity sweep, the 1024 x K x 4096 column-loc ablation shape): hot and, where
                   HBM-bound, cold (B and C rotated through more memory than the caches hold)
  cpu_baseline     the fp64 oracle (expand + dgemm) timed on the host cores on a row sample

Order of the GPU work: dense comparator, instruction probe, then 400 untimed launches of the
product kernel (`settle_launches`: the GPU's power management needs about 25 ms of a new load to
settle on a clock; the very first launch is slow, the next few run about 10 % FASTER than the
steady state), then the W warm-up steps and the K timed steps, launched back to back.  The reported
figure is therefore the steady-state throughput of a long-running job.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP16_MFMA_TFLOPS = 2500.0     # MI355X dense fp16 matrix peak
PEAK_HBM_GBS = 8000.0
CACHE_BYTES = 256 << 20            # memory-side cache; the cold runs rotate through more than this plus the L2s


def algorithmic_bytes(R, K, C, V, M, out_bytes=2):
    """Bytes the method has to move from/to HBM once: values, metadata, column-loc, C, and the rows of
    B that at least one block row selects (a row is selected by a block row with probability 4/M; with
    the few block rows of a short, very sparse matrix part of B is never read)."""
    G = K // M
    b_rows = K if M == 4 else int(round(K * (1.0 - (1.0 - 4.0 / M) ** (R // V))))
    return 2 * R * G * 2 + R * G // 2 + (R // V) * G * 4 * 2 + 2 * b_rows * C + out_bytes * R * C


def profiled_traffic(workload):
    """HBM-side bytes per launch from the committed rocprofv3 summary of this workload (a line
    `traffic_bytes_per_launch: N` in profiles/spmm_kernel_<workload>_pmc.md), or None."""
    path = os.path.join(ROOT, "profiles", f"spmm_kernel_{workload}_pmc.md")
    try:
        with open(path) as f:
            m = re.search(r"^traffic_bytes_per_launch:\s*(\d+)\s*(.*)$", f.read(), re.M)
    except OSError:
        return None, None
    if not m:
        return None, None
    return int(m.group(1)), f"profiles/{os.path.basename(path)} {m.group(2).strip()}".strip()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="gpt3",
                    help="gpt3 | bert_large | bert_base | tiny | sweep_v{V}_m{M}_c{C} | colloc_k{K}_m{M}")
    ap.add_argument("--variant", type=int, default=-1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="skip the table of the other workloads")
    ap.add_argument("--calls-only", action="store_true", help="keep the table of the other entry points, skip the other workloads")
    ap.add_argument("--all-sweep-points", action="store_true",
                    help="the table holds all 36 points of the sparsity sweep (C = 256, 2048, 8192) instead of the C = 2048 column")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--settle", type=int, default=400,
                    help="untimed launches of the product kernel before the warm-up (profiling runs use fewer)")
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
    N = 2

    def timed(fn, steps, warmup):
        """W untimed launches, then exactly `steps` launches between two synchronisations, an event
        pair around every launch.  -> wall ms per step, event ms per launch: average, median, minimum."""
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

    def timed_region(fn, steps, warmup):
        """The timed region of the headline: W untimed launches, then exactly `steps` launches back to
        back between two synchronisations, ONE event pair around the whole region (on the launch
        stream).  -> wall ms per step, event ms per launch (region / steps, launch gaps included)."""
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t_start = time.perf_counter()
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t_start) * 1e3
        return wall_ms / steps, e0.elapsed_time(e1) / steps

    def parse_workload(name):
        """-> R, K, C, V, M, sigma, (seed of A and the mask, seed of B)"""
        names = list(inputs.CONFIGS)
        if name in inputs.CONFIGS:
            R, K, C, V, M, sigma = inputs.CONFIGS[name]
            seed = inputs.config_seed(names.index(name))
            return R, K, C, V, M, sigma, (seed, seed)
        parts = dict((p[0], int(p[1:])) for p in name.split("_")[1:])
        if name.startswith("sweep_"):
            # a point of the sparsity sweep, e.g. sweep_v128_m32_c256 (the seeds of the parity tests)
            V, M, C = parts["v"], parts["m"], parts["c"]
            R, K = inputs.SWEEP_SHAPE
            seed = inputs.config_seed(4) + 7 * M + V
            return R, K, C, V, M, 1.0, (seed, seed + C)
        if name.startswith("colloc_"):
            # the shape of the paper's column-loc ablation: 1024 x K x 4096 at V = 128, 2:M
            K, M = parts["k"], parts["m"]
            seed = 900 + M + K
            return 1024, K, 4096, 128, M, 1.0, (seed, seed)
        raise SystemExit(f"bench.py: unknown workload {name}")

    def build(name):
        R, K, C, V, M, sigma, (seed_a, seed_b) = parse_workload(name)
        A_bits, mask, B_bits = inputs.gen_problem(R, K, C if seed_a == seed_b else 8, V, M, sigma, seed=seed_a)
        if seed_a != seed_b:
            B_bits = inputs.gen_B(K, C, seed=seed_b)
        A_d = torch.from_numpy(A_bits.view(np.float16)).to(dev)
        mask_d = torch.from_numpy(mask).to(dev)
        h = binding.venom_compress(A_d, mask_d, V, N, M)
        del A_d, mask_d
        B_d = torch.from_numpy(B_bits.view(np.float16)).to(dev)
        return dict(name=name, R=R, K=K, C=C, V=V, M=M, seed=seed_a, h=h, B=B_d, B_bits=B_bits)

    def rooflines(w, ms):
        R, K, C, V, M = w["R"], w["K"], w["C"], w["V"], w["M"]
        useful = 2.0 * R * C * K * N / M
        alg = algorithmic_bytes(R, K, C, V, M)
        t_mfma = useful / (PEAK_FP16_MFMA_TFLOPS * 1e12)
        t_hbm = alg / (PEAK_HBM_GBS * 1e9)
        tf = useful / (ms * 1e-3) / 1e12
        if t_mfma >= t_hbm:
            return useful, alg, {"bound": "mfma", "achieved": round(tf, 2), "peak": PEAK_FP16_MFMA_TFLOPS,
                                 "unit": "TFLOP/s", "frac": round(tf / PEAK_FP16_MFMA_TFLOPS, 4)}
        gbs = alg / (ms * 1e-3) / 1e9
        return useful, alg, {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                             "frac": round(gbs / PEAK_HBM_GBS, 4)}

    # ------------------------------------------------------------------ headline workload
    t0 = time.time()
    w = build(args.workload)
    t_gen = time.time() - t0
    R, K, C, V, M, h, B_d = w["R"], w["K"], w["C"], w["V"], w["M"], w["h"], w["B"]
    C_d = torch.empty((R, C), dtype=torch.float16, device=dev)
    dense_flop = 2.0 * R * C * K

    # dense comparator first (see the module docstring), then the instruction probe
    dense_entry = None
    if not args.no_dense:
        dense_A = binding.venom_decompress(h)     # the expanded masked matrix
        D_d = torch.empty((R, C), dtype=torch.float16, device=dev)
        dense = lambda: torch.matmul(dense_A, B_d, out=D_d)
        n_dense = max(5, min(60, int(80.0 / max(dense_flop / 1.4e12, 1e-3)) + 1))   # about 80 ms of load (1.4 PFLOP/s assumed)
        _, d_avg = timed_region(dense, n_dense, max(2, args.warmup // 5))
        dense_entry = {"ms": round(d_avg, 5), "tflops": round(dense_flop / (d_avg * 1e-3) / 1e12, 2), "launches": n_dense,
                       "kind": "torch.matmul fp16 (hipBLASLt), same R x K x C, expanded masked A"}
        del D_d, dense_A
    sink = torch.zeros(1, dtype=torch.float32, device=dev)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    probe_iters = 4000
    _, p_avg, _, _ = timed(lambda: binding.venom_probe_smfmac_rate(probe_iters, sink), 20, 3)
    measured_peak = probe_iters * 8 * 32768.0 * 16 * cus / (p_avg * 1e-3) / 1e12

    # what the memory system of this GPU sustains for plain streaming kernels (context for the
    # bandwidth-bound rows: the published 8 TB/s is not reached by any access pattern)
    cal = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()      # 1 GiB
    cal2 = torch.empty_like(cal)
    _, _, w_med, _ = timed(lambda: cal2.fill_(1.0), 10, 2)
    _, _, c_med, _ = timed(lambda: cal2.copy_(cal), 10, 2)
    hbm_cal = {"bytes": 1 << 30, "write_GBs": round((1 << 30) / (w_med * 1e-3) / 1e9, 1),
               "copy_GBs_read_plus_write": round((2 << 30) / (c_med * 1e-3) / 1e9, 1),
               "kind": "torch fill_ / copy_ on 1 GiB fp32 tensors (linear streams), median of 10"}
    del cal, cal2

    step = lambda: binding.venom_spmm(h, B_d, out=C_d, variant=args.variant)
    # The power management needs about a hundred launches (25 ms) of THIS kernel to settle on its
    # clock: the first launch after a change of load is slow, the next few are about 10 % faster than
    # the steady state.  The figure of merit is the throughput of a long-running job, so the kernel
    # runs untimed until then (reported as settle_launches); the W warm-up steps and the K timed
    # steps follow directly.
    settle_launches = max(0, args.settle)
    for _ in range(settle_launches):
        step()
    ms_wall, ms_avg = timed_region(step, args.steps, args.warmup)
    # the spread of single launches, outside the timed region (an event pair per launch leaves gaps)
    _, ms_single_avg, ms_med, ms_min = timed(step, min(args.steps, 200), 0)

    # the same launches with nothing left in the caches from the launch before: copies of the
    # compressed matrix, of B and of C rotate through more memory than the memory-side cache holds
    cold_entry = None
    if not args.no_configs and args.variant < 0:
        per = algorithmic_bytes(R, K, C, V, M)
        ncopies = int(max(3, min(8, (CACHE_BYTES + (64 << 20)) // per + 2)))
        v_e, c_e, m_e = binding.venom_export(h)
        hs = [h] + [binding.venom_import(v_e, c_e, m_e, R, K, V, N, M) for _ in range(ncopies - 1)]
        del v_e, c_e, m_e
        Bs = [B_d] + [B_d.clone() for _ in range(ncopies - 1)]
        Cs = [C_d] + [torch.empty_like(C_d) for _ in range(ncopies - 1)]
        rot = {"i": 0}

        def cold_step():
            i = rot["i"] = (rot["i"] + 1) % ncopies
            binding.venom_spmm(hs[i], Bs[i], out=Cs[i])
        _, cold_ms = timed_region(cold_step, args.steps, args.warmup)
        cold_entry = {"ms_per_step": round(cold_ms, 5), "copies": ncopies,
                      "useful_tflops": round(2.0 * R * C * K * N / M / (cold_ms * 1e-3) / 1e12, 2),
                      "kind": "compressed matrix, B and C rotated through %d copies each (%.0f MB per copy)" % (ncopies, per / 1e6)}
        del hs, Bs, Cs

    useful_flop, alg_bytes, roofline = rooflines(w, ms_avg)
    value = useful_flop / (ms_wall * 1e-3) / 1e12
    traffic, traffic_src = profiled_traffic(args.workload) if args.variant < 0 else (None, None)
    roofline["traffic"] = traffic
    roofline["traffic_source"] = traffic_src
    roofline["kernel_ms_avg"] = round(ms_avg, 5)
    roofline["timing"] = "one HIP event pair around the timed region on the launch stream, divided by the steps"
    roofline["algorithmic_bytes"] = alg_bytes
    roofline["useful_flop"] = useful_flop
    if roofline["bound"] == "mfma":
        roofline["frac_of_measured_peak"] = round(roofline["achieved"] / measured_peak, 4)

    variants = binding.venom_spmm_variants()
    out = {
        "metric": "V:N:M SpMM useful TFLOP/s (fp16)", "value": round(value, 2), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "settle_launches": settle_launches,
        "ms_per_step": round(ms_wall, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: A {R}x{K} fp16 in {V}:{N}:{M}, B {K}x{C} fp16, C fp16 (fp32 accumulate)",
                   "R": R, "K": K, "C": C, "V": V, "N": N, "M": M, "seed": w["seed"],
                   "variant": variants[args.variant] if args.variant >= 0 else "auto"},
        "dense_equivalent_tflops": round(dense_flop / (ms_wall * 1e-3) / 1e12, 2),
        "frac_of_fp16_mfma_peak_useful_wall_timed": round(value / PEAK_FP16_MFMA_TFLOPS, 4),
        "kernel_ms": {"avg": round(ms_avg, 5), "single_launch_avg": round(ms_single_avg, 5), "median": round(ms_med, 5),
                      "min": round(ms_min, 5),
                      "note": "avg: the timed region's event time / steps; the others: an event pair per launch, after the region"},
        "roofline": roofline,
        "measured_peak": {"tflops_useful": round(measured_peak, 1), "ms": round(p_avg, 4),
                          "kind": "v_smfmac_f32_32x32x32_f16 on register operands, 16 waves per compute unit, "
                                  "pseudo-random values; useful FLOP = half of the dense-equivalent count"},
    }
    if cold_entry is not None:
        out["cold_operands"] = cold_entry
    out["hbm_calibration"] = hbm_cal
    out["tables_timing"] = ("calls, configs and the dense comparators: W warm-up launches, then the stated number of launches "
                            "back to back under one HIP event pair, time / launches (throughput, like the headline)")
    if dense_entry is not None:
        dense_entry["speedup_of_spmm"] = round(dense_entry["ms"] / ms_avg, 3)
        dense_entry["ideal_speedup"] = M / N
        out["dense_gemm"] = dense_entry

    # ------------------------------------------------------------------ the other calls on the headline matrix
    if not args.no_configs and args.variant < 0:
        n = 100
        bias_d = torch.randn(R, device=dev, dtype=torch.float32).to(torch.float16)
        X_d = B_d.t().contiguous()                       # tokens x K, as a linear layer holds its activations
        Y_d = torch.empty((C, R), dtype=torch.float16, device=dev)
        scratch = torch.empty(max(2 * K * C, 16), dtype=torch.uint8, device=dev)
        calls = []

        def call_entry(name, fn, bytes_moved=None):
            _, med = timed_region(fn, n, 20)
            e = {"call": name, "ms": round(med, 5)}
            if bytes_moved is not None:
                e.update({"algorithmic_bytes": int(bytes_moved), "GBs": round(bytes_moved / (med * 1e-3) / 1e9, 1),
                          "frac_of_hbm_peak": round(bytes_moved / (med * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)})
            else:
                e["useful_tflops"] = round(useful_flop / (med * 1e-3) / 1e12, 2)
            calls.append(e)

        call_entry("venom_spmm", step)
        call_entry("venom_spmm_bias_act: bias", lambda: binding.venom_spmm(h, B_d, out=C_d, bias=bias_d))
        call_entry("venom_spmm_bias_act: bias + GELU", lambda: binding.venom_spmm(h, B_d, out=C_d, bias=bias_d, activation="gelu"))
        call_entry("venom_linear (token-major in and out, transpose of the activations included)",
                   lambda: binding.venom_linear(h, X_d, out=Y_d, scratch=scratch))
        call_entry("venom_linear: bias + GELU",
                   lambda: binding.venom_linear(h, X_d, out=Y_d, scratch=scratch, bias=bias_d, activation="gelu"))
        del X_d, Y_d, scratch
        # once-per-matrix calls on a dense matrix of the same shape: magnitude pruning, compression
        g = torch.Generator(device=dev).manual_seed(w["seed"])
        W_d = (torch.randn((R, K), generator=g, device=dev, dtype=torch.float32) * 0.02).to(torch.float16)
        pruned = binding.venom_prune(W_d, V, N, M)
        call_entry("venom_prune (dense fp16 in, mask out)", lambda: binding.venom_prune(W_d, V, N, M), 3.0 * R * K)
        ws_keep = []

        def compress_once():
            ws_keep.clear()
            ws_keep.append(binding.venom_compress(W_d, pruned[0], V, N, M))
        _, c_med = timed_region(compress_once, 10, 2)
        cb = 3.0 * R * K + 2.0 * (4.5 * R * (K // M)) + 8.0 * (R // V) * (K // M)   # A + mask in, canonical + packed arrays out
        calls.append({"call": "venom_compress (dense + mask in, canonical and packed arrays out; one host round trip)",
                      "ms": round(c_med, 5), "algorithmic_bytes": int(cb), "GBs": round(cb / (c_med * 1e-3) / 1e9, 1),
                      "frac_of_hbm_peak": round(cb / (c_med * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)})
        ws_keep.clear()
        del W_d, pruned, bias_d
        out["calls"] = calls

    # ------------------------------------------------------------------ the other workloads
    if not args.no_configs and not args.calls_only and args.workload == "gpt3" and args.variant < 0:
        names = ["tiny", "bert_base", "bert_large"]
        sweep_c = inputs.SWEEP_C if args.all_sweep_points else (2048,)
        names += [f"sweep_v{v}_m{m}_c{c}" for c in sweep_c for v in inputs.SWEEP_V for m in inputs.SWEEP_M]
        names += [f"colloc_k{k}_m{m}" for k in (4000, 16000) for m in (10, 20, 40, 100)]
        table = []
        for name in names:
            x = build(name)
            Rx, Kx, Cx = x["R"], x["K"], x["C"]
            Cx_d = torch.empty((Rx, Cx), dtype=torch.float16, device=dev)
            n = 100
            _, med = timed_region(lambda: binding.venom_spmm(x["h"], x["B"], out=Cx_d), n, 100)
            uf, ab, rf = rooflines(x, med)
            entry = {"workload": name, "R": Rx, "K": Kx, "C": Cx, "V": x["V"], "M": x["M"],
                     "ms_hot": round(med, 5), "useful_tflops": round(uf / (med * 1e-3) / 1e12, 2),
                     "bound": rf["bound"], "frac": rf["frac"], "achieved": rf["achieved"], "unit": rf["unit"]}
            if rf["bound"] == "mfma":
                entry["frac_of_measured_peak"] = round(rf["achieved"] / measured_peak, 4)
            else:
                # cold: B and C rotate through more memory than the memory-side cache and the L2s hold
                per = 2 * Kx * Cx + 2 * Rx * Cx
                nrot = min(12, (CACHE_BYTES + (64 << 20)) // per + 2)
                Bs = [x["B"]] + [x["B"].clone() for _ in range(nrot - 1)]
                Cs = [Cx_d] + [torch.empty_like(Cx_d) for _ in range(nrot - 1)]
                state = {"i": 0}

                def cold_step():
                    i = state["i"] = (state["i"] + 1) % nrot
                    binding.venom_spmm(x["h"], Bs[i], out=Cs[i])
                _, cmed = timed_region(cold_step, n, 10)
                _, _, crf = rooflines(x, cmed)
                entry.update({"ms_cold": round(cmed, 5), "frac_cold": crf["frac"], "achieved_cold": crf["achieved"],
                              "cold_buffers": int(nrot)})
                del Bs, Cs
            if not args.no_dense:
                dA = binding.venom_decompress(x["h"])
                Dx = torch.empty((Rx, Cx), dtype=torch.float16, device=dev)
                _, dmed = timed_region(lambda: torch.matmul(dA, x["B"], out=Dx), 30, 5)
                entry.update({"dense_ms": round(dmed, 5), "speedup": round(dmed / med, 3), "ideal_speedup": x["M"] / N})
                del dA, Dx
            table.append(entry)
            del x, Cx_d
        out["configs"] = table

    # ------------------------------------------------------------------ the oracle on the host cores
    if not args.no_cpu_baseline:
        from oracle import vnm_oracle as o
        v_d, c_d, m_d = binding.venom_export(h)
        torch.cuda.synchronize()
        v = v_d.cpu().numpy().view(np.uint16)
        c = c_d.cpu().numpy().view(np.uint16)
        m = m_d.cpu().numpy().view(np.uint32)
        cores = len(os.sched_getaffinity(0))
        B_bits = w["B_bits"]

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
    out["host_seconds"] = {"generate_inputs": round(t_gen, 1), "total": round(time.time() - t0, 1)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
