"""How many random samples until a wrong kernel is caught (Sec. 5.2, Fig. 2), on the CPU with
mistakes planted in a numpy model of the method (tests/mutants.py), never on the GPU.  The
sampling is the campaign's: random shape, mask, input family, seed; the verdict per sample is
the library's accuracy contract against the fp64 oracle."""
import random

import numpy as np

from oracle import ref
from paper_2403_16863_amd import inputs as I
from tests import mutants as M

O_TOL, LSE_RTOL = 3e-2, 1e-3      # bf16 contract
LENGTHS = (1, 2, 17, 33, 63, 64, 65, 100, 127, 128, 129, 191, 200, 256, 257)
FAMILIES = ("normal", "normal", "wide", "peaked", "equal_scores", "large_negative", "single_v_row")


def draw_case(rng):
    N = rng.choice(LENGTHS)
    d = rng.choice((64, 128))
    causal = rng.random() < 0.6
    fam = rng.choice(FAMILIES)
    seed = rng.randrange(1 << 30)
    if fam in ("normal", "wide"):
        w = I.Workload("m", 1, 1, N, d, causal, I.BF16, qk_sigma=2.0 if fam == "wide" else 1.0)
        qb, kb, vb = I.make_qkv(w, seed)
    else:
        qb, kb, vb = I.make_adversarial(fam, 1, 1, N, d, I.BF16, seed)
    scale = float(np.float32(1.0) / np.sqrt(np.float32(d)))
    O_ref, l_ref, _ = ref.attn_ref(qb, kb, vb, causal, scale, I.BF16)
    f = lambda b: I.bits_to_f64(b, I.BF16)[0, 0]
    return f(qb), f(kb), f(vb), causal, scale, O_ref[0, 0], l_ref[0, 0]


def caught(case, bug):
    q, k, v, causal, scale, O_ref, l_ref = case
    O, l = M.tiled_attention(q, k, v, causal, scale, bug)
    if not (np.isfinite(O).all() and np.isfinite(l).all()):
        return True
    return bool(np.max(np.abs(O - O_ref)) > O_TOL or np.max(np.abs(l - l_ref) / np.maximum(1.0, np.abs(l_ref))) > LSE_RTOL)


def first_detection(bugs, samples, seed):
    """{bug: index of the first sample that catches it (1-based), or None}; the correct method rides along."""
    rng = random.Random(seed)
    first = {b: None for b in bugs}
    for n in range(1, samples + 1):
        case = draw_case(rng)
        assert not caught(case, None), "the correct method must pass every sample"
        for b in bugs:
            if first[b] is None and caught(case, b):
                first[b] = n
    return first


def test_model_of_the_method_agrees_with_the_oracle():
    rng = random.Random(1)
    for _ in range(12):
        q, k, v, causal, scale, O_ref, l_ref = draw_case(rng)
        O, l = M.tiled_attention(q, k, v, causal, scale)
        assert np.max(np.abs(O - O_ref)) < 1e-10 and np.max(np.abs(l - l_ref)) < 1e-10


def test_planted_mistakes_are_caught_by_random_samples():
    first = first_detection(list(M.BUGS), samples=60, seed=5)
    must = ("tail_key_dropped", "no_rescale_of_O", "diag_first_key", "stale_v_tile", "lse_in_base_2")
    for b in must:
        assert first[b] is not None, f"{b} survived 60 samples"
    # the curve of Fig. 2: wrong kernels still alive after n samples never grows, and the first sample
    # alone does not catch everything (some mistakes need the right shape)
    alive = [sum(1 for b in must if first[b] > n) for n in range(0, 61)]
    assert alive == sorted(alive, reverse=True) and alive[-1] == 0
    # mistakes random testing does not see: one is harmless (a reference above the true maximum
    # changes nothing after normalisation), one needs scores hundreds above the first tile's
    # before float64 overflows -- the reason the paper calls the guarantee probabilistic
    assert first["mask_after_max"] is None and first["first_tile_only_max"] is None


# ---- second workload

GEMM_MS = (1, 7, 31, 32, 33, 64, 65, 100)
GEMM_NS = (8, 16, 24, 40, 64, 72)
GEMM_KS = (8, 16, 32, 40, 64, 104, 128, 136, 256, 264, 512, 520)


def draw_gemm_case(rng):
    Mm, N, K = rng.choice(GEMM_MS), rng.choice(GEMM_NS), rng.choice(GEMM_KS)
    fam = rng.choice(I.GEMM_FAMILIES)
    slope = rng.choice((0.01, 0.2, 0.0, -0.5))
    ab, bb = I.make_gemm(Mm, N, K, I.F16, rng.randrange(1 << 30), fam)
    x, _ = ref.gemm_lrelu_ref(ab, bb, slope, I.F16)
    sabs, _ = ref.gemm_lrelu_ref(ab & np.uint16(0x7FFF), bb & np.uint16(0x7FFF), 1.0, I.F16)
    tol = 1.01 * 2.0 ** -11 * np.abs(x) + 2.0 * K * 2.0 ** -24 * sabs * max(1.0, abs(slope)) + 2.0 ** -25
    return I.bits_to_f64(ab, I.F16), I.bits_to_f64(bb, I.F16), slope, x, tol


def gemm_caught(case, bug):
    a, b, slope, x, tol = case
    c = M.tiled_gemm_lrelu(a, b, slope, bug)
    return bool(not np.isfinite(c).all() or (np.abs(c - x) > tol).any())


def gemm_first_detection(samples=80, seed=11):
    rng = random.Random(seed)
    first = {b: None for b in M.GEMM_BUGS}
    for n in range(1, samples + 1):
        case = draw_gemm_case(rng)
        assert not gemm_caught(case, None), "the correct method must pass every sample"
        for b in first:
            if first[b] is None and gemm_caught(case, b):
                first[b] = n
    return first


def test_gemm_model_and_its_planted_mistakes():
    first = gemm_first_detection()
    for b in ("k_tail_dropped", "k_tail_not_zeroed", "worker_sum_misses_last", "row_tail_wraps", "relu_instead_of_leaky",
              "b_tile_transposed_within_8"):
        assert first[b] is not None, f"{b} survived 80 samples"
    assert first["relu_instead_of_leaky"] <= 5 and first["b_tile_transposed_within_8"] <= 5
    # harmless by construction: rounding keeps the sign, and slope * 0 = 0
    assert first["slope_on_negative_zero"] is None


if __name__ == "__main__":   # prints the curve:  python -m tests.test_sample_curve [samples] [seed]
    import sys
    samples = int(sys.argv[1]) if len(sys.argv) > 1 else 300
    seed = int(sys.argv[2]) if len(sys.argv) > 2 else 0
    first = first_detection(list(M.BUGS), samples, seed)
    for b, n in sorted(first.items(), key=lambda kv: (kv[1] is None, kv[1])):
        print(f"{b:24s} first caught at sample {n}   ({M.BUGS[b][0]}; shows when: {M.BUGS[b][1]})")
    for n in (1, 2, 5, 10, 20, 50, 100, 200, samples):
        if n <= samples:
            print(f"after {n:4d} samples: {sum(1 for v in first.values() if v is None or v > n)} of {len(first)} mutants not caught")
    for b, n in sorted(gemm_first_detection(samples).items(), key=lambda kv: (kv[1] is None, kv[1])):
        print(f"gemm {b:28s} first caught at sample {n}   ({M.GEMM_BUGS[b][0]}; shows when: {M.GEMM_BUGS[b][1]})")
