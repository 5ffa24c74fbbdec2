"""Pins for the batched vector-matrix oracle (the paper's Case Study 2,
C[m, n] = sum_k A[m, k] B[m, n, k]). None of the expected values below comes from the oracle."""
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import gemm_oracle as orc
from paper_2512_09196_amd import workloads as wl


def bits(x):
    return wl.f64_to_bf16_bits(np.asarray(x, dtype=np.float64))


def vals(b):
    return wl.bf16_bits_to_f32(b).astype(np.float64)


def test_exact_rational_brute_force_on_small_cases():
    rng = np.random.default_rng(5)
    for (M, N, K) in ((1, 1, 1), (2, 3, 4), (3, 5, 7), (4, 2, 9)):
        A = bits(rng.normal(0, 1, (M, K)))
        B = bits(rng.uniform(-1, 1, (M, N, K)))
        c, s = orc.batched_vecmat(A, B)
        a, b = vals(A), vals(B)
        for m in range(M):
            for n in range(N):
                exact = sum(Fraction(a[m, k]) * Fraction(b[m, n, k]) for k in range(K))
                exact_abs = sum(abs(Fraction(a[m, k]) * Fraction(b[m, n, k])) for k in range(K))
                # bf16 x bf16 products are exact in double; K <= 9 additions lose at most K ulps
                assert abs(Fraction(c[m, n]) - exact) <= K * Fraction(2) ** -52 * max(exact_abs, Fraction(1, 10 ** 30))
                assert abs(Fraction(s[m, n]) - exact_abs) <= K * Fraction(2) ** -52 * exact_abs


def test_ones_vector_gives_row_sums_of_each_matrix():
    M, N, K = 3, 17, 130
    B = wl.uniform_bf16(21, 1, (M, N, K), 0.25)
    A = bits(np.ones((M, K)))
    c, s = orc.batched_vecmat(A, B)
    b = vals(B)
    for m in range(M):
        for n in range(N):
            want = math.fsum(b[m, n, :])               # exactly rounded, independent of the oracle's order
            assert abs(c[m, n] - want) <= K * 2.0 ** -52 * math.fsum(np.abs(b[m, n, :])) + 1e-300
            assert abs(s[m, n] - math.fsum(np.abs(b[m, n, :]))) <= K * 2.0 ** -52 * s[m, n]


def test_delta_matrices_pick_single_elements_of_the_vector():
    # B[m, n, k] = 1 where k == (3 m + n) mod K: C[m, n] = A[m, (3 m + n) mod K]. A wrong batch index,
    # a swap of n and k, or the vector of another row all give another element.
    M, N, K = 4, 11, 7
    A = wl.normal_bf16(3, 0, (M, K), 1.0)
    B = np.zeros((M, N, K))
    for m in range(M):
        for n in range(N):
            B[m, n, (3 * m + n) % K] = 1.0
    c, s = orc.batched_vecmat(A, bits(B))
    a = vals(A)
    for m in range(M):
        for n in range(N):
            assert c[m, n] == a[m, (3 * m + n) % K]
            assert s[m, n] == abs(a[m, (3 * m + n) % K])


def test_one_row_is_a_plain_matrix_vector_product():
    N, K = 37, 300
    A = wl.normal_bf16(8, 0, (1, K), 1.0)
    B = wl.uniform_bf16(8, 1, (1, N, K), 0.1)
    c, _ = orc.batched_vecmat(A, B)
    want = vals(B)[0] @ vals(A)[0]                    # library routine on the special case
    assert np.allclose(c[0], want, rtol=0, atol=K * 2.0 ** -50)


def test_integer_operands_give_exact_integers():
    M, N, K = 5, 9, 64
    A = wl.small_int_bf16(4, 0, (M, K))
    B = wl.small_int_bf16(4, 1, (M, N, K))
    c, s = orc.batched_vecmat(A, B)
    a, b = vals(A).astype(np.int64), vals(B).astype(np.int64)
    want = np.einsum("mk,mnk->mn", a, b)
    assert np.array_equal(c, want.astype(np.float64))
    assert np.array_equal(s, np.einsum("mk,mnk->mn", np.abs(a), np.abs(b)).astype(np.float64))


def test_power_of_two_scaling_is_exact_and_rows_are_independent():
    M, N, K = 3, 6, 50
    A = wl.normal_bf16(12, 0, (M, K), 1.0)
    B = wl.uniform_bf16(12, 1, (M, N, K), 0.5)
    c, _ = orc.batched_vecmat(A, B)
    c4, _ = orc.batched_vecmat(bits(vals(A) * 4.0), B)
    assert np.array_equal(c4, 4.0 * c)
    # changing row 1 of A changes row 1 of C only
    A2 = A.copy()
    A2[1] = bits(-vals(A)[1])
    c2, _ = orc.batched_vecmat(A2, B)
    assert np.array_equal(c2[0], c[0]) and np.array_equal(c2[2], c[2]) and np.array_equal(c2[1], -c[1])


def test_empty_and_degenerate_sizes():
    c, s = orc.batched_vecmat(np.zeros((2, 0), np.uint16), np.zeros((2, 3, 0), np.uint16))
    assert c.shape == (2, 3) and not c.any() and not s.any()
    c, _ = orc.batched_vecmat(np.zeros((0, 4), np.uint16), np.zeros((0, 3, 4), np.uint16))
    assert c.shape == (0, 3)
    with pytest.raises(ValueError):
        orc.batched_vecmat(np.zeros((2, 4), np.uint16), np.zeros((2, 3, 5), np.uint16))


def test_vecmat_generator_is_deterministic_and_has_the_stated_distributions():
    w = wl.VECMAT_WORKLOADS["V1"]
    A, B = wl.make_vecmat(w.M, w.N, w.K, w.seed)
    A2, B2 = wl.make_vecmat(w.M, w.N, w.K, w.seed)
    assert A.dtype == np.uint16 and B.shape == (w.M, w.N, w.K)
    assert np.array_equal(A, A2) and np.array_equal(B, B2)
    a, b = vals(A), vals(B)
    assert abs(a.mean()) < 0.05 and abs(a.std() - 1.0) < 0.05
    lim = w.K ** -0.5
    assert np.abs(b).max() <= lim * (1 + 2.0 ** -8) and abs(b.std() - lim / math.sqrt(3.0)) < 0.02 * lim   # (rounding to bf16 may step past the limit by half an ulp)
    assert w.flops == 2 * w.M * w.N * w.K and w.algorithmic_bytes == 2 * (w.M * w.K + w.M * w.N * w.K) + 4 * w.M * w.N
