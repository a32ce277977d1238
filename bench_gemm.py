#!/usr/bin/env python3
"""Benchmark of the second workload, fused GEMM + LeakyReLU (Sec. 5, Table 3: M, N, K = 512, 512,
2048, binary16), on one MI355X.  The paper's metric for it is the kernel's latency.

A step is one launch of the whole path (tile loads through LDS, MFMA, cross-wave sum, activation,
rounding, store) on seeded synthetic A, B already resident in device memory.  Prints ONE JSON line.

  python bench_gemm.py [--steps K] [--warmup W] [--variant ID] [--dtype f16|bf16] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# Bytes per launch that cross the L2 boundary, from `rocprofv3 --pmc FETCH_SIZE` and `--pmc WRITE_SIZE`
# runs of this script scaled by the same counters on a 256 MiB device copy (FETCH_SIZE counts
# 2 KiB, WRITE_SIZE 1 KiB); default variant, binary16.  Written up under profiles/.
MEASURED_HBM_BYTES = (6185.0 * 2.0 + 512.0 * 1.0) * 1024


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--variant", type=int, default=None)
    ap.add_argument("--dtype", choices=("f16", "bf16"), default="f16")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench_gemm.py measures one GPU; nothing here runs on more than one")

    import numpy as np
    import torch
    from paper_2403_16863_amd import gemm, inputs as I
    if not torch.cuda.is_available():
        sys.exit("bench_gemm.py needs a GPU")
    dtype = I.F16 if args.dtype == "f16" else I.BF16
    M, N, K, slope = I.GEMM_M, I.GEMM_N, I.GEMM_K, I.GEMM_SLOPE
    ab, bb = I.make_gemm(M, N, K, dtype, seed=0)
    tdt = torch.float16 if dtype == I.F16 else torch.bfloat16
    a, b = (torch.from_numpy(x.view(np.int16)).to("cuda").view(tdt) for x in (ab, bb))
    c = torch.empty((M, N), dtype=tdt, device="cuda")
    variant = gemm.gemm_lrelu_default_variant(M, N, K) if args.variant is None else args.variant

    stream = torch.cuda.current_stream()
    for _ in range(args.warmup):
        gemm.gemm_lrelu_variant(a, b, c, slope, variant)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(args.steps):
        gemm.gemm_lrelu_variant(a, b, c, slope, variant)
    e1.record(stream)
    torch.cuda.synchronize()
    wall_us = (time.perf_counter() - t0) / args.steps * 1e6
    # the same launches issued by the library itself, without the interpreter between them
    dev_us = gemm.gemm_lrelu_time(a, b, c, slope, variant, 50, args.steps) / args.steps * 1e3
    # what one launch costs on this device before it does any work: a single-tile problem
    ta, tb = a[:32, :8].contiguous(), b[:8, :32].contiguous()
    tc = torch.empty((32, 32), dtype=tdt, device="cuda")
    floor_us = gemm.gemm_lrelu_time(ta, tb, tc, slope, variant, 50, args.steps) / args.steps * 1e3

    alg_bytes = 2.0 * (M * K + K * N + M * N)          # every operand element once, 16 bits each
    flops = 2.0 * M * N * K
    out = {
        "metric": "gemm_lrelu_latency", "value": dev_us, "unit": "us", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": dev_us * 1e-3, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": f"gemm_lrelu M{M} N{N} K{K} {args.dtype}", "slope": slope, "variant": variant,
                   "knobs": dict(zip(gemm.KNOB_NAMES, gemm.gemm_lrelu_variant_knobs(variant)))},
        "tflops": flops / dev_us / 1e6,
        "latency_us_with_python_launch": wall_us,
        "launch_floor_us": floor_us,
        "roofline": {"bound": "hbm", "achieved": alg_bytes / dev_us / 1e3, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": alg_bytes / dev_us / 1e3 / HBM_PEAK_GBS, "traffic": MEASURED_HBM_BYTES if (args.variant is None and dtype == I.F16) else None,
                     "algorithmic_bytes": alg_bytes,
                     "note": "launches back to back; a launch that does no work takes launch_floor_us of it"},
    }
    if not args.no_cpu_baseline:
        from oracle import ref
        t0 = time.perf_counter()
        x, used = ref.gemm_lrelu_ref(ab, bb, float(np.float32(slope)), dtype)
        cpu_s = time.perf_counter() - t0
        err = float(np.abs(c.to(torch.float64).cpu().numpy() - x).max())
        out["cpu_baseline"] = {"value": cpu_s * 1e6, "unit": "us", "cores": used, "kind": "oracle",
                               "sample": "the whole problem, once", "max_abs_err_vs_oracle": err}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
