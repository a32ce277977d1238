#!/usr/bin/env python3
"""Benchmark of the fused attention forward on one MI355X.

A step is one pass of the whole hot path (one attn_fwd launch: Q tile load, K/V
streaming through LDS, Q.K^T on MFMA, mask, online softmax, P.V on MFMA, epilogue)
over one batch of seeded synthetic Q/K/V that already sits in HBM.  Prints ONE JSON
line.  FLOP convention: 4*B*H*N^2*d, halved for causal.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload IDX] [--variant ID]
                  [--no-cpu-baseline] [--no-mfma-ceiling] [--all]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_PEAK_TFLOPS = 2500.0   # MI355X dense bf16/fp16 MFMA peak (published)

# HBM bytes per launch of the default variant, from `rocprofv3 --pmc FETCH_SIZE` and
# `--pmc WRITE_SIZE` runs scaled by the same counters on a 256 MiB device copy (FETCH_SIZE
# counts 2 KiB, WRITE_SIZE 1 KiB); the runs and numbers are written up under profiles/.
MEASURED_HBM_BYTES = {
    "cfg2": (137699 * 2.0 + 75787.1 * 1.0) * 1024,
    "cfg3": (334452 * 2.0 + 148992 * 1.0) * 1024,
}


def device_tensors(w, seed):
    import numpy as np
    import torch
    from paper_2403_16863_amd import inputs as I
    qb, kb, vb = I.make_qkv(w, seed)
    tdt = torch.bfloat16 if w.dtype == I.BF16 else torch.float16
    q, k, v = (torch.from_numpy(a.view(np.int16)).to("cuda").view(tdt) for a in (qb, kb, vb))
    out = torch.empty_like(q)
    lse = torch.empty(q.shape[:3], dtype=torch.float32, device="cuda")
    return (qb, kb, vb), (q, k, v, out, lse)


def time_steps(A, w, tensors, variant, warmup, steps):
    """Wall clock over exactly `steps` launches bracketed by synchronize, plus the
    average launch duration from HIP events recorded on the launch stream."""
    import torch
    q, k, v, out, lse = tensors
    stream = torch.cuda.current_stream()
    for _ in range(warmup):
        A.attn_fwd_variant(q, k, v, out, lse, w.causal, w.scale, variant)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(steps):
        A.attn_fwd_variant(q, k, v, out, lse, w.causal, w.scale, variant)
    e1.record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    return (t1 - t0) / steps, e0.elapsed_time(e1) * 1e-3 / steps


def calibrate_copy(nbytes=256 << 20, reps=5):
    """A plain device-to-device copy of known size, for scaling the FETCH_SIZE / WRITE_SIZE
    counters of a `rocprofv3 --pmc` run (it reads nbytes and writes nbytes per launch)."""
    import torch
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(reps):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"calibrate_copy_bytes": nbytes, "launches": reps}), flush=True)


def cpu_baseline(w, bits, out, lse, budget_s=15.0):
    """The oracle as it stands, timed on this machine's host cores on a bounded row sample
    of the same workload; also returns the GPU-vs-oracle error on that sample."""
    import numpy as np
    from oracle import ref
    from paper_2403_16863_amd import inputs as I
    qb, kb, vb = bits

    def row_flops(rows):
        i = rows % w.N
        vis = (i + 1) if w.causal else np.full_like(i, w.N)
        return float(np.sum(4.0 * w.d * vis))

    # size the sample from a probe that is large enough to amortise the per-head decode
    total_rows = w.B * w.H * w.N
    nprobe = min(total_rows, 4096)
    probe = I.sample_rows(w, nprobe, seed=99)
    t0 = time.perf_counter()
    ref.attn_ref(qb, kb, vb, w.causal, w.scale, w.dtype, rows=probe)
    t_probe = max(time.perf_counter() - t0, 1e-4)
    n = int(min(total_rows, max(nprobe, nprobe * budget_s / t_probe)))
    rows = I.sample_rows(w, n, seed=100)
    t0 = time.perf_counter()
    O_ref, l_ref, threads = ref.attn_ref(qb, kb, vb, w.causal, w.scale, w.dtype, rows=rows)
    dt = time.perf_counter() - t0
    fl = row_flops(rows)
    O = out.double().cpu().numpy().reshape(-1, w.d)[rows]
    l = lse.double().cpu().numpy().reshape(-1)[rows]
    err_o = float(np.max(np.abs(O - O_ref)))
    err_l = float(np.max(np.abs(l - l_ref) / np.maximum(1.0, np.abs(l_ref))))
    base = {"value": fl / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{len(rows)} of {total_rows} query rows of {w.name} (stratified over heads, "
                      f"first/last/tile-edge rows included), {fl / 1e9:.2f} GFLOP in {dt:.2f} s"}
    parity = {"rows": int(len(rows)), "max_abs_err_O": err_o, "max_rel_err_lse": err_l,
              "tol_O": 3e-2 if w.dtype == I.BF16 else 1e-2, "tol_lse": 1e-3}
    return base, parity


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", type=int, default=2, help="index into the benchmark configs (default 2)")
    ap.add_argument("--variant", type=int, default=None, help="schedule variant id (default: library default)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-mfma-ceiling", action="store_true",
                    help="skip the MFMA-only kernel that measures the sustained matrix-core rate of this device")
    ap.add_argument("--all", action="store_true", help="also time the other configs (reported under 'others')")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a 256 MiB device copy (counter calibration for rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1")

    import torch
    import paper_2403_16863_amd as A
    from paper_2403_16863_amd import inputs as I
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        calibrate_copy()
        return

    w = I.WORKLOADS[args.workload]
    bits, tensors = device_tensors(w, seed=args.workload)
    variant = args.variant if args.variant is not None else A.attn_default_variant(w.N, w.d, w.dtype, w.causal)
    wall_s, evt_s = time_steps(A, w, tensors, variant, args.warmup, args.steps)
    tflops = w.flops / wall_s / 1e12
    achieved = w.flops / evt_s / 1e12

    result = {
        "metric": "attention fwd TFLOP/s and % of MFMA bf16/fp16 peak on 1 MI355X",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall_s * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": I.DTYPE_NAMES[w.dtype], "data": "synthetic",
        "config": {"workload": w.label, "flop_convention": "4*B*H*N^2*d, halved for causal",
                   "variant": variant, "variant_desc": A.attn_variant_desc(variant),
                   "pct_of_mfma_peak": 100.0 * tflops / MFMA_PEAK_TFLOPS},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / MFMA_PEAK_TFLOPS,
                     "traffic": MEASURED_HBM_BYTES.get(w.name) if args.variant is None else None},
    }
    if not args.no_mfma_ceiling:
        # what the MFMA pipe alone sustains on this device (about 0.3 s each): context for frac
        tf_c, ghz_c = A.attn_mfma_ceiling(False)
        tf_r, ghz_r = A.attn_mfma_ceiling(True)
        result["roofline"]["mfma_only_kernel"] = {
            "constant_operands": {"TFLOP/s": tf_c, "core_GHz": ghz_c},
            "random_operands": {"TFLOP/s": tf_r, "core_GHz": ghz_r},
            "frac_of_random_operand_rate": achieved / tf_r if tf_r > 0 else None,
            "note": "bf16 MFMAs from registers only; with random operands the device lowers its clock"}
    if not args.no_cpu_baseline:
        base, parity = cpu_baseline(w, bits, tensors[3], tensors[4])
        result["cpu_baseline"] = base
        result["parity_vs_oracle"] = parity
    if args.all:
        others = {}
        for idx, ow in enumerate(I.WORKLOADS):
            if idx == args.workload:
                continue
            _, t = device_tensors(ow, seed=idx)
            ov = A.attn_default_variant(ow.N, ow.d, ow.dtype, ow.causal)
            ws, es = time_steps(A, ow, t, ov, args.warmup, args.steps)
            others[ow.label] = {"ms": ws * 1e3, "TFLOP/s": ow.flops / ws / 1e12,
                                "pct_of_mfma_peak": 100.0 * ow.flops / es / 1e12 / MFMA_PEAK_TFLOPS}
            del t
            torch.cuda.empty_cache()
        result["others"] = others
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
