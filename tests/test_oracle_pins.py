"""Pins for the CPU oracle: checks against things other than the oracle itself.

The paper prints no worked attention example (it names the kernel, Sec. 1 / Sec. 5,
and the [batch, heads, seq, head_dim] format, Table 2 caption), so the pins are the
mathematics: bit-pattern decoding against numpy's own types, a differently written
brute force, closed forms, invariants and a library composition.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import ref
from paper_2403_16863_amd import inputs as I

HERE = os.path.dirname(os.path.abspath(__file__))


def bits(x, dtype):
    return I.f32_to_bits(np.asarray(x, dtype=np.float32), dtype)


def rand_bits(shape, dtype, seed, sigma=1.0):
    g = np.random.default_rng(seed)
    return bits(g.standard_normal(shape) * sigma, dtype)


# ----------------------------------------------------------------- decoding

@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
def test_decode_all_bit_patterns(dtype):
    allbits = np.arange(65536, dtype=np.uint16)
    want = I.bits_to_f64(allbits, dtype)
    got = np.array([ref.decode(int(b), dtype) for b in allbits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))  # -0.0 too


def test_bf16_rounding_is_nearest_even():
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: goes to even (1.0);
    # 1 + 3*2^-8 is a tie between 1+2^-7 and 1+2^-6: goes to even (1 + 2^-6).
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20], dtype=np.float32)
    got = I.bits_to_f64(I.f32_to_bits(x, I.BF16), I.BF16)
    assert got.tolist() == [1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7]


# -------------------------------------------------------------- brute force

def brute_force(q, k, v, causal, scale):
    """Differently written: whole N x N matrix in long double, no max
    subtraction, normalise by direct division, matrix product at the end."""
    B, H, N, d = q.shape
    ql, kl, vl = (a.astype(np.longdouble) for a in (q, k, v))
    O = np.zeros((B, H, N, d), dtype=np.longdouble)
    lse = np.zeros((B, H, N), dtype=np.longdouble)
    for b in range(B):
        for h in range(H):
            S = np.longdouble(scale) * (ql[b, h] @ kl[b, h].T)
            E = np.exp(S)
            if causal:
                E = np.tril(E)
            Z = E.sum(axis=1)
            O[b, h] = (E / Z[:, None]) @ vl[b, h]
            lse[b, h] = np.log(Z)
    return O, lse


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("shape", [(1, 1, 1, 1), (1, 1, 2, 3), (2, 3, 7, 4), (1, 2, 8, 5), (1, 1, 33, 16)])
def test_brute_force_tiny(shape, causal, dtype):
    qb = rand_bits(shape, dtype, 1)
    kb = rand_bits(shape, dtype, 2)
    vb = rand_bits(shape, dtype, 3)
    scale = 0.37
    O, lse, _ = ref.attn_ref(qb, kb, vb, causal, scale, dtype)
    q, k, v = (I.bits_to_f64(a, dtype) for a in (qb, kb, vb))
    Ob, lb = brute_force(q, k, v, causal, scale)
    assert np.max(np.abs(O - Ob.astype(np.float64))) <= 1e-12
    assert np.max(np.abs(lse - lb.astype(np.float64))) <= 1e-12


# -------------------------------------------------------------- closed forms

def test_golden_ln2_example():
    rowsf = []
    with open(os.path.join(HERE, "golden", "closed_form_ln2.txt")) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                mode, row, num, den, lnarg = line.split()
                rowsf.append((mode, int(row), Fraction(int(num), int(den)), int(lnarg)))
    q = bits(np.ones((1, 1, 3, 1)), I.F16)
    k = bits(np.array([0.0, 1.0, 2.0]).reshape(1, 1, 3, 1), I.F16)
    v = bits(np.array([7.0, 14.0, -7.0]).reshape(1, 1, 3, 1), I.F16)
    res = {m: ref.attn_ref(q, k, v, m == "causal", math.log(2.0), I.F16) for m in ("full", "causal")}
    assert len(rowsf) == 6
    for mode, row, o_exact, lnarg in rowsf:
        O, lse, _ = res[mode]
        assert abs(O[0, 0, row, 0] - float(o_exact)) <= 1e-13
        assert abs(lse[0, 0, row] - math.log(lnarg)) <= 1e-13


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
def test_n1_output_is_v(dtype):
    shape = (2, 2, 1, 8)
    qb, kb, vb = (rand_bits(shape, dtype, s) for s in (4, 5, 6))
    for causal in (False, True):
        O, lse, _ = ref.attn_ref(qb, kb, vb, causal, 0.5, dtype)
        q, k, v = (I.bits_to_f64(a, dtype) for a in (qb, kb, vb))
        assert np.array_equal(O, v)
        assert np.allclose(lse[..., 0], 0.5 * np.sum(q * k, axis=-1)[..., 0], rtol=0, atol=1e-14)


def test_n2_is_logistic_sigmoid():
    dtype = I.F16
    shape = (1, 1, 2, 6)
    qb, kb, vb = (rand_bits(shape, dtype, s) for s in (7, 8, 9))
    scale = 0.8
    O, lse, _ = ref.attn_ref(qb, kb, vb, False, scale, dtype)
    q, k, v = (I.bits_to_f64(a, dtype)[0, 0] for a in (qb, kb, vb))
    for i in range(2):
        z = scale * float(q[i] @ (k[0] - k[1]))
        w0 = 1.0 / (1.0 + math.exp(-z))          # weight of key 0
        want = w0 * v[0] + (1.0 - w0) * v[1]
        assert np.max(np.abs(O[0, 0, i] - want)) <= 1e-14
        x0, x1 = scale * float(q[i] @ k[0]), scale * float(q[i] @ k[1])
        assert abs(lse[0, 0, i] - (max(x0, x1) + math.log1p(math.exp(-abs(x0 - x1))))) <= 1e-14


@pytest.mark.parametrize("causal", [False, True])
def test_zero_q_gives_uniform_average(causal):
    dtype = I.BF16
    B, H, N, d = 1, 2, 19, 4
    qb = bits(np.zeros((B, H, N, d)), dtype)
    kb, vb = rand_bits((B, H, N, d), dtype, 10), rand_bits((B, H, N, d), dtype, 11)
    O, lse, _ = ref.attn_ref(qb, kb, vb, causal, 1.0, dtype)
    v = I.bits_to_f64(vb, dtype)
    for i in range(N):
        n = i + 1 if causal else N
        assert np.max(np.abs(O[:, :, i] - v[:, :, :n].mean(axis=2))) <= 1e-14
        assert np.max(np.abs(lse[:, :, i] - math.log(n))) <= 1e-14


def test_one_hot_scores_are_exact():
    # Q rows and K rows are unit vectors: scores are exactly 0 or `scale`.
    dtype = I.F16
    N = d = 5
    eye = np.eye(N).reshape(1, 1, N, d)
    qb, kb = bits(eye, dtype), bits(eye, dtype)
    vb = rand_bits((1, 1, N, d), dtype, 12)
    s = 3.0
    O, lse, _ = ref.attn_ref(qb, kb, vb, False, s, dtype)
    v = I.bits_to_f64(vb, dtype)[0, 0]
    Z = math.exp(s) + (N - 1)
    for i in range(N):
        w = np.full(N, 1.0 / Z)
        w[i] = math.exp(s) / Z
        assert np.max(np.abs(O[0, 0, i] - w @ v)) <= 1e-14
        assert abs(lse[0, 0, i] - math.log(Z)) <= 1e-14


# ---------------------------------------------------------------- invariants

@pytest.mark.parametrize("causal", [False, True])
def test_probability_rows_sum_to_one(causal):
    dtype = I.F16
    shape = (1, 2, 40, 8)
    qb, kb = rand_bits(shape, dtype, 13, 2.0), rand_bits(shape, dtype, 14, 2.0)
    for row in (0, 1, 39, 40, 57, 79):
        p = ref.attn_ref_probs(qb, kb, causal, 0.35, dtype, row)
        assert abs(p.sum() - 1.0) <= 1e-12
        assert (p >= 0).all()
        if causal:
            assert (p[(row % 40) + 1:] == 0).all()


def test_probs_entry_point_agrees_with_lse():
    dtype = I.BF16
    shape = (1, 1, 23, 8)
    qb, kb, vb = (rand_bits(shape, dtype, s) for s in (15, 16, 17))
    scale = 0.6
    O, lse, _ = ref.attn_ref(qb, kb, vb, False, scale, dtype)
    q, k, v = (I.bits_to_f64(a, dtype)[0, 0] for a in (qb, kb, vb))
    for i in (0, 11, 22):
        p = ref.attn_ref_probs(qb, kb, False, scale, dtype, i)
        x = scale * (k @ q[i])
        assert np.max(np.abs(p - np.exp(x - lse[0, 0, i]))) <= 1e-13
        assert np.max(np.abs(p @ v - O[0, 0, i])) <= 1e-13


@pytest.mark.parametrize("causal", [False, True])
def test_constant_v_gives_constant_output(causal):
    dtype = I.F16
    shape = (1, 2, 31, 8)
    qb, kb = rand_bits(shape, dtype, 18), rand_bits(shape, dtype, 19)
    vb = bits(np.full(shape, -1.75), dtype)
    O, _, _ = ref.attn_ref(qb, kb, vb, causal, 0.4, dtype)
    assert np.max(np.abs(O + 1.75)) <= 1e-12


def test_joint_kv_permutation_non_causal():
    dtype = I.BF16
    shape = (2, 2, 29, 8)
    qb, kb, vb = (rand_bits(shape, dtype, s) for s in (20, 21, 22))
    perm = np.random.default_rng(23).permutation(shape[2])
    O1, l1, _ = ref.attn_ref(qb, kb, vb, False, 0.3, dtype)
    O2, l2, _ = ref.attn_ref(qb, kb[:, :, perm].copy(), vb[:, :, perm].copy(), False, 0.3, dtype)
    assert np.max(np.abs(O1 - O2)) <= 1e-12
    assert np.max(np.abs(l1 - l2)) <= 1e-12
    # and it does matter when only K is permuted (guards against ignoring K order)
    O3, _, _ = ref.attn_ref(qb, kb[:, :, perm].copy(), vb, False, 0.3, dtype)
    assert np.max(np.abs(O1 - O3)) > 1e-3


def test_causal_row_equals_full_attention_on_prefix():
    dtype = I.F16
    B, H, N, d = 1, 2, 21, 8
    qb, kb, vb = (rand_bits((B, H, N, d), dtype, s) for s in (24, 25, 26))
    Oc, lc, _ = ref.attn_ref(qb, kb, vb, True, 0.45, dtype)
    for i in (0, 1, 7, 20):
        n = i + 1
        Of, lf, _ = ref.attn_ref(qb[:, :, :n].copy(), kb[:, :, :n].copy(), vb[:, :, :n].copy(),
                                 False, 0.45, dtype)
        assert np.max(np.abs(Oc[:, :, i] - Of[:, :, i])) <= 1e-13
        assert np.max(np.abs(lc[:, :, i] - lf[:, :, i])) <= 1e-13
    v = I.bits_to_f64(vb, dtype)
    assert np.array_equal(Oc[:, :, 0], v[:, :, 0])        # row 0 sees only key 0


def test_key_shift_moves_lse_only():
    # K <- K + 1 u^T adds scale*q.u to every score of a row: O unchanged, lse shifted.
    # Values sit on a 1/8 grid so K + u is exactly representable in binary16.
    dtype = I.F16
    g = np.random.default_rng(27)
    shape = (1, 1, 17, 4)
    q = g.integers(-16, 17, size=shape) / 8.0
    k = g.integers(-16, 17, size=shape) / 8.0
    v = g.integers(-16, 17, size=shape) / 8.0
    u = g.integers(-8, 9, size=(1, 1, 1, 4)) / 8.0
    scale = 0.25
    for causal in (False, True):
        O1, l1, _ = ref.attn_ref(bits(q, dtype), bits(k, dtype), bits(v, dtype), causal, scale, dtype)
        O2, l2, _ = ref.attn_ref(bits(q, dtype), bits(k + u, dtype), bits(v, dtype), causal, scale, dtype)
        assert np.max(np.abs(O1 - O2)) <= 1e-12
        shift = scale * np.sum(q * u, axis=-1)
        assert np.max(np.abs((l2 - l1) - shift)) <= 1e-12


def test_scale_is_applied_to_scores_not_probabilities():
    dtype = I.F16
    shape = (1, 1, 9, 4)
    qb, kb, vb = (rand_bits(shape, dtype, s) for s in (28, 29, 30))
    # doubling the scale equals doubling Q (exact in binary16)
    q2 = bits(2.0 * I.bits_to_f64(qb, dtype), dtype)
    O1, l1, _ = ref.attn_ref(qb, kb, vb, False, 0.5, dtype)
    O2, l2, _ = ref.attn_ref(q2, kb, vb, False, 0.25, dtype)
    assert np.max(np.abs(O1 - O2)) <= 1e-13 and np.max(np.abs(l1 - l2)) <= 1e-13
    O0, l0, _ = ref.attn_ref(qb, kb, vb, False, 0.0, dtype)   # scale 0: uniform
    assert np.max(np.abs(l0 - math.log(9))) <= 1e-14


# ------------------------------------------------- library composition check

@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("causal", [False, True])
def test_against_torch_fp64_composition(causal, dtype):
    torch = pytest.importorskip("torch")
    w = I.Workload("t", 2, 3, 150, 64, causal, dtype, qk_sigma=2.0)
    qb, kb, vb = I.make_qkv(w, seed=31)
    O, lse, _ = ref.attn_ref(qb, kb, vb, causal, w.scale, dtype)
    q, k, v = (torch.from_numpy(I.bits_to_f64(a, dtype)) for a in (qb, kb, vb))
    S = (q @ k.transpose(-1, -2)) * w.scale
    if causal:
        S = S.masked_fill(torch.ones(w.N, w.N, dtype=torch.bool).triu(1), float("-inf"))
    Ot = torch.softmax(S, dim=-1) @ v
    lt = torch.logsumexp(S, dim=-1)
    assert np.max(np.abs(O - Ot.numpy())) <= 1e-12
    assert np.max(np.abs(lse - lt.numpy())) <= 1e-12


# ------------------------------------------------------------ interface bits

def test_row_subset_matches_full_and_threads_do_not_matter():
    dtype = I.BF16
    w = I.Workload("t", 2, 2, 70, 16, True, dtype)
    qb, kb, vb = I.make_qkv(w, seed=32)
    O, lse, used1 = ref.attn_ref(qb, kb, vb, True, w.scale, dtype, nthreads=1)
    assert used1 == 1
    O4, lse4, used4 = ref.attn_ref(qb, kb, vb, True, w.scale, dtype, nthreads=4)
    assert used4 == 4
    assert np.array_equal(O, O4) and np.array_equal(lse, lse4)
    rows = np.array([0, 69, 70, 139, 200, 279, 5], dtype=np.int64)
    Os, ls, _ = ref.attn_ref(qb, kb, vb, True, w.scale, dtype, rows=rows, nthreads=3)
    assert np.array_equal(Os, O.reshape(-1, 16)[rows])
    assert np.array_equal(ls, lse.reshape(-1)[rows])


def test_bad_arguments_are_rejected():
    qb = rand_bits((1, 1, 4, 4), I.F16, 33)
    with pytest.raises(ValueError):
        ref.attn_ref(qb, qb, qb, False, 1.0, 2)                       # unknown dtype
    with pytest.raises(ValueError):
        ref.attn_ref(qb, qb, qb, False, 1.0, I.F16, rows=np.array([4]))  # row out of range


def test_large_scores_do_not_overflow():
    dtype = I.F16
    shape = (1, 1, 6, 4)
    qb = bits(np.full(shape, 200.0), dtype)
    kb = bits(np.random.default_rng(34).integers(-3, 4, size=shape) * 50.0, dtype)
    vb = rand_bits(shape, dtype, 35)
    O, lse, _ = ref.attn_ref(qb, kb, vb, False, 1.0, dtype)
    assert np.isfinite(O).all() and np.isfinite(lse).all()
    k = I.bits_to_f64(kb, dtype)[0, 0]
    x = 200.0 * k.sum(axis=1)
    j = np.flatnonzero(x == x.max())
    v = I.bits_to_f64(vb, dtype)[0, 0]
    assert np.max(np.abs(O[0, 0, 0] - v[j].mean(axis=0))) <= 1e-12    # winner(s) take all
