"""Randomised test campaign of the library's default kernels against the fp64 oracle (the
probabilistic testing of Sec. 4.2 / Sec. 5.2, with the oracle in the place of the unmodified
kernel).  Every sample draws a shape, a dtype, a mask, an input family and a seed; the
number of samples comes from ATTN_CAMPAIGN_SAMPLES (default 120: a few seconds).  Run as a
script for a long campaign:  ATTN_CAMPAIGN_SAMPLES=5000 python -m pytest tests/test_gpu_campaign.py -m gpu -s
With ATTN_CAMPAIGN_ALL_VARIANTS=1 every sample also draws one of the schedule variants built for
its head dimension, instead of the library default (by default every fourth sample does).
Tolerance on O: the absolute one of the target statement (1e-2 binary16, 3e-2 bfloat16) as long as
the largest |V| of the sample is inside the range for which the accuracy bound 2 u max|V| stays
below it (10 and 3.8), that bound beyond (tests.gpu_util.o_tol); lse: 1e-3 relative.
"""
import os
import random
import time

import numpy as np
import pytest

from oracle import ref
from paper_2403_16863_amd import inputs as I
from tests.gpu_util import O_TOL, LSE_RTOL, o_tol, run_gpu

FAMILIES = ("normal", "normal", "normal", "wide", "peaked", "equal_scores", "large_negative",
            "single_v_row", "signed_zero", "max_finite_v", "rising_scores")
# sequence lengths around every tile boundary of the shipped variants, plus odd ones
LENGTHS = (1, 2, 17, 31, 32, 33, 63, 64, 65, 100, 127, 128, 129, 191, 192, 193, 255, 256, 257, 300, 383, 384,
           385, 511, 512, 513, 640, 777, 1000, 1024, 1025)


def draw(rng):
    d = rng.choice((64, 128))
    dtype = rng.choice((I.F16, I.BF16))
    causal = rng.random() < 0.6
    N = rng.choice(LENGTHS)
    B = rng.choice((1, 1, 2, 3))
    H = rng.choice((1, 2, 3, 5, 8))
    if B * H * N > 16384:                       # keeps one oracle call well under a second
        B, H = 1, max(1, 8192 // N)
    return B, H, N, d, dtype, causal, rng.choice(FAMILIES), rng.randrange(1 << 30)


@pytest.mark.gpu
def test_campaign_against_oracle():
    samples = int(os.environ.get("ATTN_CAMPAIGN_SAMPLES", "120"))
    rng = random.Random(int(os.environ.get("ATTN_CAMPAIGN_SEED", "2024")))
    worst_o, worst_l, worst_abs, t0 = 0.0, 0.0, 0.0, time.time()
    worst_what = ""
    by_family = {}
    trace = os.environ.get("ATTN_CAMPAIGN_TRACE")  # file that names the sample in flight, for a run that dies
    all_variants = os.environ.get("ATTN_CAMPAIGN_ALL_VARIANTS") == "1"
    import paper_2403_16863_amd as A
    vrng = random.Random(rng.randrange(1 << 30))     # its own stream: the draws above stay what they were
    by_variant = {}
    print(f"campaign: {samples} samples to draw", flush=True)
    for n in range(samples):
        B, H, N, d, dtype, causal, fam, seed = draw(rng)
        if fam in ("normal", "wide"):
            w = I.Workload("c", B, H, N, d, causal, dtype, qk_sigma=2.0 if fam == "wide" else 1.0,
                           v_dist="uniform" if fam == "wide" else "normal")
            qb, kb, vb = I.make_qkv(w, seed)
        else:
            qb, kb, vb = I.make_adversarial(fam, B, H, N, d, dtype, seed)
        scale = float(np.float32(1.0) / np.sqrt(np.float32(d)))
        O_ref, l_ref, _ = ref.attn_ref(qb, kb, vb, causal, scale, dtype)
        if trace:
            with open(trace, "w") as f:
                f.write(f"sample {n}: B{B} H{H} N{N} d{d} dtype{dtype} causal{causal} {fam} seed{seed}\n")
        variant = None
        if all_variants or n % 4 == 3:
            variant = vrng.choice([v for v in range(A.attn_num_variants()) if A.attn_variant_supported(v, d, dtype, causal)])
        by_variant[variant] = by_variant.get(variant, 0) + 1
        O, l = run_gpu(qb, kb, vb, causal, scale, dtype, variant=variant)
        tol = o_tol(dtype, np.abs(I.bits_to_f64(vb, dtype)).max())  # the absolute tolerance, or 2 u max|V| where that is larger
        what = f"sample {n}: B{B} H{H} N{N} d{d} dtype{dtype} causal{causal} {fam} seed{seed} variant{variant}"
        assert np.isfinite(O).all() and np.isfinite(l).all(), what
        eo = float(np.max(np.abs(O - O_ref)))
        el = float(np.max(np.abs(l - l_ref) / np.maximum(1.0, np.abs(l_ref))))
        assert eo <= tol, f"{what}: max|dO| = {eo:.3e} > {tol:.3e}"
        assert el <= LSE_RTOL, f"{what}: lse error {el:.3e}"
        if eo / tol > worst_o:
            worst_o, worst_what = eo / tol, what
        if fam != "max_finite_v":
            worst_abs = max(worst_abs, eo / O_TOL[dtype])
        worst_l = max(worst_l, el / LSE_RTOL)
        by_family[fam] = by_family.get(fam, 0) + 1
        if (n + 1) % 250 == 0:
            print(f"campaign: {n + 1} samples passed, {time.time() - t0:.0f} s", flush=True)
    print(f"campaign: {samples} samples passed in {time.time() - t0:.1f} s; worst error as a fraction of the "
          f"tolerance: O {worst_o:.3f} ({worst_what}), lse {worst_l:.3f}; worst O error over the fixed absolute "
          f"tolerance, all families but max_finite_v: {worst_abs:.3f}; families {by_family}; "
          f"variants (None = library default) {dict(sorted(by_variant.items(), key=lambda kv: -1 if kv[0] is None else kv[0]))}", flush=True)


@pytest.mark.gpu
def test_gemm_campaign_against_oracle():
    """The same for the second workload: shape (every size a multiple of 8 where the boundary asks for
    it, around the 32-wide tile and the 32/64/128/256/512-wide k ranges), dtype, slope, input family,
    variant and seed at random; element-wise against the fp64 oracle with the tolerance derived in
    tests/test_gpu_gemm.py.  GEMM_CAMPAIGN_SAMPLES sets the count (default 60)."""
    from paper_2403_16863_amd import gemm
    from tests.test_gpu_gemm import check, run_gpu
    samples = int(os.environ.get("GEMM_CAMPAIGN_SAMPLES", "60"))
    rng = random.Random(int(os.environ.get("ATTN_CAMPAIGN_SEED", "2024")) + 1)
    ms = (1, 2, 17, 31, 32, 33, 63, 64, 65, 100, 127, 128, 129, 200, 255, 256, 257, 300, 512)
    ns = (8, 16, 24, 32, 40, 56, 64, 72, 96, 120, 128, 136, 256, 264, 512)
    ks = (8, 16, 24, 32, 40, 56, 64, 72, 120, 128, 136, 248, 256, 264, 504, 512, 520, 1000, 1024, 1032, 2048)
    nv = gemm.gemm_lrelu_num_variants()
    worst, t0 = 0.0, time.time()
    print(f"gemm campaign: {samples} samples to draw", flush=True)
    for n in range(samples):
        M, N, K = rng.choice(ms), rng.choice(ns), rng.choice(ks)
        dtype = rng.choice((I.F16, I.BF16))
        fam = rng.choice(I.GEMM_FAMILIES)
        if fam == "large" and dtype == I.F16:
            K = min(K, 1024)
        slope = rng.choice((0.01, 0.01, 0.2, 0.0, 1.0, -0.5))
        variant = rng.choice((None, rng.randrange(nv)))
        seed = rng.randrange(1 << 30)
        ab, bb = I.make_gemm(M, N, K, dtype, seed, fam)
        what = f"gemm sample {n}: M{M} N{N} K{K} dtype{dtype} {fam} slope{slope} variant{variant} seed{seed}"
        c = run_gpu(ab, bb, slope, dtype, variant)
        worst = max(worst, check(c, ab, bb, slope, dtype, what))
        if (n + 1) % 250 == 0:
            print(f"gemm campaign: {n + 1} samples passed, {time.time() - t0:.0f} s", flush=True)
    print(f"gemm campaign: {samples} samples passed in {time.time() - t0:.1f} s; worst error as a fraction of the "
          f"tolerance: {worst:.3f}", flush=True)


@pytest.mark.gpu
def test_largest_finite_binary16_v_never_overflows():
    """O is a convex combination of V values, so with V at the largest finite binary16 value the
    exact output stays finite; P rounded upwards may put the computed one half a unit in the last
    place above it, which must be stored as the largest finite value, not as infinity.  First the
    sample of a random campaign that found this (seed 141421, sample 69835), on every variant; then
    the sharpest form: every V element equal to +65504 (or -65504), so every output element is
    exactly that value and any net upward rounding of P would overflow."""
    import paper_2403_16863_amd as A
    big = 65504.0
    scale = float(np.float32(1.0) / np.sqrt(np.float32(64)))
    qb, kb, vb = I.make_adversarial("max_finite_v", 1, 3, 256, 64, I.F16, 598254998)
    O_ref, l_ref, _ = ref.attn_ref(qb, kb, vb, True, scale, I.F16)
    variants = [None] + [v for v in range(A.attn_num_variants()) if A.attn_variant_supported(v, 64, I.F16, True)]
    for variant in variants:
        O, l = run_gpu(qb, kb, vb, True, scale, I.F16, variant=variant)
        assert np.isfinite(O).all() and np.isfinite(l).all(), f"variant {variant}"
        assert float(np.max(np.abs(O - O_ref))) <= o_tol(I.F16, big), f"variant {variant}"
        assert float(np.max(np.abs(l - l_ref) / np.maximum(1.0, np.abs(l_ref)))) <= LSE_RTOL, f"variant {variant}"
    for d in (64, 128):
        for causal in (True, False):
            for sign in (1.0, -1.0):
                w = I.Workload("c", 2, 4, 193, d, causal, I.F16)
                qb, kb, vb = I.make_qkv(w, 11 + d)
                vb = I.f32_to_bits(np.full((2, 4, 193, d), sign * big, dtype=np.float32), I.F16)
                sc = float(np.float32(1.0) / np.sqrt(np.float32(d)))
                for variant in [None] + [v for v in range(A.attn_num_variants()) if A.attn_variant_supported(v, d, I.F16, causal)]:
                    O, _ = run_gpu(qb, kb, vb, causal, sc, I.F16, variant=variant)
                    assert np.isfinite(O).all(), f"d {d} causal {causal} sign {sign} variant {variant}"
                    # 65504 or the binary16 value below it (65472)
                    assert float(np.max(np.abs(O - sign * big))) <= 32.0, f"d {d} causal {causal} sign {sign} variant {variant}"
