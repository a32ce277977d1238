"""Pins of the GEMM + LeakyReLU oracle (oracle/gemm_ref.cpp) to things other than itself: exact
rational arithmetic on tiny cases, closed forms, algebraic identities and a library routine."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import ref
from paper_2403_16863_amd import inputs as I


def bits(x, dtype=I.F16):
    return I.f32_to_bits(np.asarray(x, dtype=np.float32), dtype)


def vals(b, dtype=I.F16):
    return I.bits_to_f64(b, dtype)


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
def test_exact_rational_brute_force(dtype):
    g = np.random.default_rng(3)
    for (M, N, K) in ((1, 1, 1), (2, 3, 4), (5, 4, 7), (3, 5, 1)):
        a, b = bits(g.standard_normal((M, K)), dtype), bits(g.standard_normal((K, N)), dtype)
        av, bv = vals(a, dtype), vals(b, dtype)
        slope = 0.125
        C, _ = ref.gemm_lrelu_ref(a, b, slope, dtype)
        for i in range(M):
            for j in range(N):
                s = sum(Fraction(float(av[i, k])) * Fraction(float(bv[k, j])) for k in range(K))   # exact
                want = s if s >= 0 else Fraction(slope) * s
                assert abs(C[i, j] - float(want)) <= 1e-14 * max(1.0, abs(float(want)))


def test_identity_and_ones_closed_forms():
    g = np.random.default_rng(4)
    K = 37
    b = bits(g.standard_normal((K, 11)))
    C, _ = ref.gemm_lrelu_ref(bits(np.eye(K)), b, 0.01, I.F16)             # A = I: C = leaky_relu(B)
    bv = vals(b)
    assert np.array_equal(C, np.where(bv >= 0, bv, 0.01 * bv))
    C, _ = ref.gemm_lrelu_ref(bits(np.ones((6, K))), bits(np.ones((K, 9))), 0.3, I.F16)
    assert np.array_equal(C, np.full((6, 9), float(K)))                    # all ones: C = K
    C, _ = ref.gemm_lrelu_ref(bits(-np.ones((6, K))), bits(np.ones((K, 9))), 0.25, I.F16)
    assert np.array_equal(C, np.full((6, 9), -0.25 * K))                   # negative branch: slope * (-K)
    C, _ = ref.gemm_lrelu_ref(bits(np.zeros((2, 3))), bits(np.ones((3, 2))), 0.5, I.F16)
    assert np.array_equal(C, np.zeros((2, 2)))


def test_slope_one_is_a_plain_product_and_matches_the_library_routine():
    g = np.random.default_rng(5)
    a, b = bits(g.standard_normal((33, 300))), bits(g.standard_normal((300, 29)))
    C, _ = ref.gemm_lrelu_ref(a, b, 1.0, I.F16)
    want = vals(a) @ vals(b)                                                # numpy float64 matmul
    assert np.max(np.abs(C - want)) <= 1e-12 * np.max(np.abs(want))
    C0, _ = ref.gemm_lrelu_ref(a, b, 0.0, I.F16)                            # slope 0: ReLU
    assert np.max(np.abs(C0 - np.maximum(want, 0.0))) <= 1e-12 * np.max(np.abs(want))
    Cn, _ = ref.gemm_lrelu_ref(a, b, -2.0, I.F16)                           # any real slope is legal
    assert np.max(np.abs(Cn - np.where(want >= 0, want, -2.0 * want))) <= 1e-11 * np.max(np.abs(want))


def test_algebraic_identities():
    g = np.random.default_rng(6)
    a, b = bits(g.standard_normal((17, 64))), bits(g.standard_normal((64, 13)))
    slope = 0.01
    C, _ = ref.gemm_lrelu_ref(a, b, slope, I.F16)
    # transposition: leaky_relu(A B)^T = leaky_relu(B^T A^T)
    Ct, _ = ref.gemm_lrelu_ref(np.ascontiguousarray(b.T), np.ascontiguousarray(a.T), slope, I.F16)
    assert np.max(np.abs(Ct.T - C)) <= 1e-12
    # positive homogeneity with an exact scale: leaky_relu((2A) B) = 2 leaky_relu(A B)
    C2, _ = ref.gemm_lrelu_ref(bits(2.0 * vals(a)), b, slope, I.F16)
    assert np.array_equal(C2, 2.0 * C)
    # sign flip swaps the branches: leaky_relu(-x) = -slope * leaky_relu(x) / 1 on x > 0, -x/slope... checked elementwise
    Cm, _ = ref.gemm_lrelu_ref(bits(-vals(a)), b, slope, I.F16)
    P, _ = ref.gemm_lrelu_ref(a, b, 1.0, I.F16)
    assert np.array_equal(Cm, np.where(-P >= 0, -P, slope * -P))
    # a permutation of the inner index changes nothing but the order of summation
    perm = g.permutation(64)
    Cp, _ = ref.gemm_lrelu_ref(np.ascontiguousarray(a[:, perm]), np.ascontiguousarray(b[perm, :]), slope, I.F16)
    assert np.max(np.abs(Cp - C)) <= 1e-12
    # thread count does not matter
    C1, used = ref.gemm_lrelu_ref(a, b, slope, I.F16, nthreads=1)
    assert used == 1 and np.array_equal(C1, C)


def test_rejects_bad_arguments():
    with pytest.raises(ValueError):
        ref.gemm_lrelu_ref(bits(np.ones((2, 3))), bits(np.ones((4, 2))), 0.1, I.F16)
    with pytest.raises(ValueError):
        ref.gemm_lrelu_ref(bits(np.ones((2, 3))), bits(np.ones((3, 2))), 0.1, 7)
