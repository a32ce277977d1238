#!/usr/bin/env python3
"""Benchmark of the fused attention forward on one MI355X.

A step is one pass of the whole hot path (one attn_fwd launch: Q tile load, K/V
streaming through LDS, Q.K^T on MFMA, mask, online softmax, P.V on MFMA, epilogue)
over one batch of seeded synthetic Q/K/V that already sits in HBM.  Prints ONE JSON
line.  FLOP convention: 4*B*H*N^2*d, halved for causal.

The timed workload is the largest single-GPU configuration (index 3: B1 H32 N16384 d128
causal bf16); the other target shape (index 2) and the second workload (GEMM + LeakyReLU)
are timed in the same process and reported under "others".

Before the timed region the kernel is launched, untimed, until a fixed amount of GPU time
has passed (config.settle_launches says how many launches that was): the device lowers its
clock under the switching activity of real data over the first tens of milliseconds, and a
short run would otherwise time that transient instead of the sustained rate.  --warmup and
--steps are used exactly as passed, after that phase.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload IDX] [--variant ID]
                  [--no-cpu-baseline] [--no-ceilings] [--no-others] [--all]
"""
import argparse
import glob
import json
import os
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_PEAK_TFLOPS = 2500.0   # MI355X dense bf16/fp16 MFMA peak (published)
HBM_PEAK_GBS = 8000.0
SETTLE_GPU_SECONDS = 0.4    # untimed launches before warm-up and the timed steps

# HBM bytes per launch of the default variant, from `rocprofv3 --pmc FETCH_SIZE` and
# `--pmc WRITE_SIZE` runs scaled by the same counters on a 256 MiB device copy (FETCH_SIZE
# counts 2 KiB, WRITE_SIZE 1 KiB); the runs and numbers are written up under profiles/.
# These are constants taken from those profiles, not measured in this run.
PROFILE_HBM_BYTES = {
    "cfg2": ((141957 * 2.0 + 66560 * 1.0) * 1024, "profiles/attn_fwd_cfg2_B2_H32_N4096_d128_causal_bf16.md"),
    "cfg3": ((311040 * 2.0 + 133120 * 1.0) * 1024, "profiles/attn_fwd_cfg3_B1_H32_N16384_d128_causal_bf16.md"),
}
GEMM_PROFILE_HBM_BYTES = ((6185.0 * 2.0 + 512.0 * 1.0) * 1024, "profiles/gemm_lrelu_M512_N512_K2048_f16.md")


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


class DeviceSampler(threading.Thread):
    """Reads the GPU's core clock and socket power from sysfs while the timed region runs
    (no child process, no device call).  Values are None where the files are not readable."""

    def __init__(self, period_s=0.01):
        super().__init__(daemon=True)
        self.period = period_s
        self.stop_flag = threading.Event()
        self.clock_mhz, self.power_w = [], []
        self.freq_files, self.power_files, self.cap_w = [], [], None
        devs = []
        try:
            import torch
            pr = torch.cuda.get_device_properties(0)
            bus = f"{getattr(pr, 'pci_domain_id', 0):04x}:{pr.pci_bus_id:02x}:{pr.pci_device_id:02x}.0"
            devs = glob.glob(f"/sys/bus/pci/devices/{bus}")
        except Exception:
            devs = []
        self.source = "sysfs (pp_dpm_sclk, hwmon) of the PCI device of cuda:0" if devs else "sysfs (pp_dpm_sclk, hwmon), busiest card"
        if not devs:
            devs = glob.glob("/sys/class/drm/card*/device")
        for dev in devs:
            f = os.path.join(dev, "pp_dpm_sclk")       # lines "n: <MHz>Mhz", the current one marked with *
            if os.path.exists(f):
                self.freq_files.append(f)
            for r in glob.glob(os.path.join(dev, "hwmon", "hwmon*")):
                for name in ("power1_average", "power1_input"):
                    pf = os.path.join(r, name)
                    if os.path.exists(pf):
                        self.power_files.append(pf)
                        break
                cap = self._read(os.path.join(r, "power1_cap"))
                if cap:
                    self.cap_w = cap / 1e6

    @staticmethod
    def _read(path):
        try:
            with open(path) as fh:
                return float(fh.read().strip())
        except Exception:
            return None

    @staticmethod
    def _read_sclk(path):
        try:
            with open(path) as fh:
                for line in fh:
                    if "*" in line:
                        return float(line.split(":")[1].lower().replace("mhz", "").replace("*", "").strip()) * 1e6
        except Exception:
            pass
        return None

    def run(self):
        while not self.stop_flag.is_set():
            fr = [x for x in (self._read_sclk(f) for f in self.freq_files) if x]
            pw = [x for x in (self._read(f) for f in self.power_files) if x]
            if fr:
                self.clock_mhz.append(max(fr) / 1e6)
            if pw:
                self.power_w.append(max(pw) / 1e6)
            time.sleep(self.period)

    def result(self):
        import numpy as np
        return {"core_clock_GHz": float(np.median(self.clock_mhz)) / 1e3 if self.clock_mhz else None,
                "socket_power_W": float(np.median(self.power_w)) if self.power_w else None,
                "power_cap_W": self.cap_w, "samples": max(len(self.clock_mhz), len(self.power_w)), "source": self.source}


def settle(A, w, tensors, variant, gpu_seconds=SETTLE_GPU_SECONDS):
    """Untimed launches until `gpu_seconds` of GPU time have passed; returns (launches, GPU ms)."""
    import torch
    q, k, v, out, lse = tensors
    stream = torch.cuda.current_stream()
    launches, gpu_ms = 0, 0.0
    while gpu_ms < gpu_seconds * 1e3:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(10):
            A.attn_fwd_variant(q, k, v, out, lse, w.causal, w.scale, variant)
        e1.record(stream)
        torch.cuda.synchronize()
        gpu_ms += e0.elapsed_time(e1)
        launches += 10
    return launches, gpu_ms


def time_steps(A, w, tensors, variant, warmup, steps, sample_device=False):
    """Wall clock over exactly `steps` launches bracketed by synchronize, and the average launch
    duration from one pair of HIP events recorded on the launch stream around the same launches.
    Afterwards, outside the timed region, up to 50 more launches are bracketed one by one (an
    event between every two launches adds a few microseconds each) for the median and minimum."""
    import numpy as np
    import torch
    q, k, v, out, lse = tensors
    stream = torch.cuda.current_stream()
    for _ in range(warmup):
        A.attn_fwd_variant(q, k, v, out, lse, w.causal, w.scale, variant)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    sampler = DeviceSampler() if sample_device else None
    torch.cuda.synchronize()
    if sampler:
        sampler.start()
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(steps):
        A.attn_fwd_variant(q, k, v, out, lse, w.causal, w.scale, variant)
    e1.record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    if sampler:
        sampler.stop_flag.set()
        sampler.join()
    per_launch = np.array(A.attn_time_variant(q, k, v, out, lse, w.causal, w.scale, variant, 0, min(steps, 50)))
    return {"wall_s": (t1 - t0) / steps, "evt_s": e0.elapsed_time(e1) * 1e-3 / steps,
            "launch_ms": {"median": float(np.median(per_launch)), "min": float(per_launch.min()), "max": float(per_launch.max()),
                          "launches": int(len(per_launch)), "note": "each launch between its own pair of events, after the timed region"},
            "device": sampler.result() if sampler else None}


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


def ceilings(A, achieved):
    """What the matrix cores alone and the vector ALU alone sustain on this device (about a
    second in all): context for roofline.frac, and the second ceiling of the path."""
    tf_c, ghz_c = A.attn_mfma_ceiling(False)
    tf_r, ghz_r = A.attn_mfma_ceiling(True)
    mfma = {"constant_operands": {"TFLOP/s": tf_c, "core_GHz": ghz_c},
            "random_operands": {"TFLOP/s": tf_r, "core_GHz": ghz_r},
            "frac_of_random_operand_rate": achieved / tf_r if tf_r > 0 else None,
            "note": "bf16 MFMAs from registers only; with random operands the device lowers its clock"}
    mix = {"note": "the tile loop's own instruction mix and nothing else (random operands, two waves per SIMD, "
                   "no tile loads, barriers, masks or item boundaries): the ceiling of the loop body at this device's power limit"}
    for mode, name in ((0, "mfma_only"), (1, "mfma_and_lds_reads"), (2, "mfma_lds_reads_and_softmax_arithmetic")):
        tf, ghz = A.attn_mix_ceiling(mode)
        mix[name] = {"TFLOP/s": tf, "core_GHz": ghz}
    mix["frac_of_full_mix_rate"] = achieved / mix["mfma_lds_reads_and_softmax_arithmetic"]["TFLOP/s"]
    # the same mix in the ping-pong form of the default kernels (one wave of a SIMD in an MFMA cluster, the
    # other in a vector cluster): what that structure costs before any tile load, mask or item boundary
    import torch
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    for mode, name in ((3, "pingpong_form_two_barriers_per_tile"), (4, "pingpong_form_one_barrier_per_tile")):
        tf, ghz = A.attn_mix_ceiling(mode, 40000)
        mix[name] = {"TFLOP/s": tf, "core_GHz": ghz,
                     "clocks_per_tile": (ghz * 1e9 * 32 * 32768.0 * 8 * cus / (tf * 1e12)) if tf > 0 else None,
                     "mfma_clocks_per_tile": 2048}
    mix["frac_of_pingpong_form_rate"] = achieved / mix["pingpong_form_one_barrier_per_tile"]["TFLOP/s"]
    mfma["loop_body_mix_kernel"] = mix
    valu = {"mix": "per score element 1 fma + 1 exp2 + 1 add + 1/2 conversion to 16 bit, from registers, no packed fp32",
            "note": "an element stands for 4*d flops of the two contractions: implied ceilings below"}
    for wps in (1, 2, 3):
        eps, ghz = A.attn_valu_ceiling(wps)
        valu[f"waves_per_simd_{wps}"] = {"Gelements/s": eps / 1e9, "core_GHz": ghz,
                                         "implied_TFLOP/s_d64": eps * 4 * 64 / 1e12,
                                         "implied_TFLOP/s_d128": eps * 4 * 128 / 1e12}
    return mfma, valu


def gemm_leg(steps=5000, warmup=200, with_oracle=True):
    """The second workload (GEMM + LeakyReLU, M, N, K = 512, 512, 2048, binary16): latency per launch,
    the cost of a launch that does no work, the algorithmic-bytes roofline, and the oracle's time."""
    import numpy as np
    import torch
    from paper_2403_16863_amd import gemm, inputs as I
    M, N, K, slope = I.GEMM_M, I.GEMM_N, I.GEMM_K, I.GEMM_SLOPE
    ab, bb = I.make_gemm(M, N, K, I.F16, seed=0)
    a, b = (torch.from_numpy(x.view(np.int16)).to("cuda").view(torch.float16) for x in (ab, bb))
    c = torch.empty((M, N), dtype=torch.float16, device="cuda")
    variant = gemm.gemm_lrelu_default_variant(M, N, K)
    dev_us = gemm.gemm_lrelu_time(a, b, c, slope, variant, warmup, steps) / steps * 1e3
    ta, tb = a[:32, :8].contiguous(), b[:8, :32].contiguous()
    tc = torch.empty((32, 32), dtype=torch.float16, device="cuda")
    floor_us = gemm.gemm_lrelu_time(ta, tb, tc, slope, variant, warmup, steps) / steps * 1e3
    alg_bytes = 2.0 * (M * K + K * N + M * N)
    leg = {"workload": f"gemm_lrelu M{M} N{N} K{K} f16, slope {slope}", "variant": variant,
           "latency_us": dev_us, "launch_floor_us": floor_us, "TFLOP/s": 2.0 * M * N * K / dev_us / 1e6,
           "steps": steps, "warmup": warmup,
           "roofline": {"bound": "hbm", "achieved": alg_bytes / dev_us / 1e3, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": alg_bytes / dev_us / 1e3 / HBM_PEAK_GBS, "algorithmic_bytes": alg_bytes,
                        "traffic": GEMM_PROFILE_HBM_BYTES[0], "traffic_source": GEMM_PROFILE_HBM_BYTES[1] + " constant"}}
    if with_oracle:
        from oracle import ref
        t0 = time.perf_counter()
        x, used = ref.gemm_lrelu_ref(ab, bb, float(np.float32(slope)), I.F16)
        cpu_s = time.perf_counter() - t0
        leg["cpu_baseline"] = {"value": cpu_s * 1e6, "unit": "us", "cores": used, "kind": "oracle",
                               "sample": "the whole problem, once"}
        leg["max_abs_err_vs_oracle"] = float(np.abs(c.to(torch.float64).cpu().numpy() - x).max())
    return leg


def search_summary(name):
    """Best searched schedule against the hand-written default, from the ranking the search
    tool stored for this workload (paper_2403_16863_amd/search_store/); None if there is none."""
    path = os.path.join(ROOT, "paper_2403_16863_amd", "search_store", f"ranking_{name}.json")
    if not os.path.exists(path):
        return None
    with open(path) as fh:
        r = json.load(fh)
    return {"best_variant": r.get("best_variant"), "best_vs_default": r.get("best_vs_default"),
            "best_vs_variant0": r.get("best_vs_variant0"), "default_variant": r.get("default_variant"),
            "measured_on": r.get("measured_on"), "source": os.path.relpath(path, ROOT) + " (stored ranking, not measured in this run)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", type=int, default=3, help="index into the benchmark configs (default 3, the largest)")
    ap.add_argument("--variant", type=int, default=None, help="schedule variant id (default: library default)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ceilings", "--no-mfma-ceiling", dest="no_ceilings", action="store_true",
                    help="skip the MFMA-only and vector-ALU-only kernels that measure this device's sustained rates")
    ap.add_argument("--no-others", action="store_true", help="skip the other target shape and the GEMM leg")
    ap.add_argument("--no-settle", action="store_true", help="skip the untimed settle phase (for profiler runs)")
    ap.add_argument("--all", action="store_true", help="also time the three small configs (reported under 'others')")
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
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    # Sec. 4.1: what the stored searches found better than the default (by more than the timing
    # noise) is deployed, and is then what attn_fwd, and this bench, launch.
    from paper_2403_16863_amd import deploy
    deployed = deploy.deploy_stored_rankings()

    def run_workload(idx, variant=None, sample_device=False):
        w = I.WORKLOADS[idx]
        bits, tensors = device_tensors(w, seed=idx)
        var = variant if variant is not None else A.attn_deployed(w.N, w.d, w.dtype, w.causal)[1]
        settled = (0, 0.0) if args.no_settle else settle(A, w, tensors, var)
        t = time_steps(A, w, tensors, var, args.warmup, args.steps, sample_device=sample_device)
        return w, bits, tensors, var, settled, t

    w, bits, tensors, variant, settled, t = run_workload(args.workload, args.variant, sample_device=True)
    tflops = w.flops / t["wall_s"] / 1e12
    achieved = w.flops / t["evt_s"] / 1e12
    traffic = PROFILE_HBM_BYTES.get(w.name) if args.variant is None else None

    result = {
        "metric": "attention fwd TFLOP/s and % of MFMA bf16/fp16 peak on 1 MI355X",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": t["wall_s"] * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": I.DTYPE_NAMES[w.dtype], "data": "synthetic",
        "config": {"workload": w.label, "flop_convention": "4*B*H*N^2*d, halved for causal",
                   "variant": variant, "variant_desc": A.attn_variant_desc(variant),
                   "pct_of_mfma_peak": 100.0 * tflops / MFMA_PEAK_TFLOPS,
                   "settle_launches": settled[0], "settle_gpu_ms": settled[1],
                   "settle_note": "untimed launches before --warmup and --steps, until the device's clock has settled",
                   "compute_units": cus, "launch_ms": t["launch_ms"], "device_during_timed_region": t["device"]},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / MFMA_PEAK_TFLOPS,
                     "traffic": traffic[0] if traffic else None,
                     "traffic_source": (traffic[1] + " constant (profiled once, not measured in this run)") if traffic else None},
    }
    if not args.no_ceilings:
        result["roofline"]["mfma_only_kernel"], result["roofline"]["valu_only_kernel"] = ceilings(A, achieved)
    if not args.no_cpu_baseline:
        base, parity = cpu_baseline(w, bits, tensors[3], tensors[4])
        result["cpu_baseline"] = base
        result["parity_vs_oracle"] = parity
    result["search"] = search_summary(w.name)
    if result["search"] is not None:
        result["search"]["deployed"] = deployed
    del tensors, bits
    torch.cuda.empty_cache()

    others = {}
    if not args.no_others:
        idxs = [i for i in ((2, 3) if not args.all else range(len(I.WORKLOADS))) if i != args.workload]
        for idx in idxs:
            ow, obits, otensors, ov, osettled, ot = run_workload(idx)
            ach = ow.flops / ot["evt_s"] / 1e12
            otr = PROFILE_HBM_BYTES.get(ow.name)
            others[ow.name] = {"workload": ow.label, "variant": ov, "ms_per_step": ot["wall_s"] * 1e3,
                               "TFLOP/s": ow.flops / ot["wall_s"] / 1e12, "launch_ms": ot["launch_ms"],
                               "settle_launches": osettled[0],
                               "roofline": {"bound": "mfma", "achieved": ach, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                                            "frac": ach / MFMA_PEAK_TFLOPS, "traffic": otr[0] if otr else None,
                                            "traffic_source": (otr[1] + " constant") if otr else None},
                               "search": search_summary(ow.name)}
            if not args.no_cpu_baseline and idx in (2, 3):
                _, oparity = cpu_baseline(ow, obits, otensors[3], otensors[4], budget_s=4.0)
                others[ow.name]["parity_vs_oracle"] = oparity
            del otensors, obits
            torch.cuda.empty_cache()
        others["gemm_lrelu"] = gemm_leg(with_oracle=not args.no_cpu_baseline)
    if others:
        result["others"] = others
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
