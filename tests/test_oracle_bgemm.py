"""Pins for the oracle of the batched transposed-operand product (the paper's Case Study 3,
C[b, m, n] = sum_k A[b, k, m] B[b, k, n]). None of the expected values comes from the oracle."""
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
    rng = np.random.default_rng(11)
    for (nb, M, N, K) in ((1, 1, 1, 1), (2, 3, 4, 5), (3, 2, 5, 7)):
        A = bits(rng.normal(0, 1, (nb, K, M)))
        B = bits(rng.uniform(-1, 1, (nb, K, N)))
        c, s = orc.batched_gemm_tn(A, B)
        a, b = vals(A), vals(B)
        for i in range(nb):
            for m in range(M):
                for n in range(N):
                    exact = sum(Fraction(a[i, k, m]) * Fraction(b[i, k, n]) for k in range(K))
                    exact_abs = sum(abs(Fraction(a[i, k, m]) * Fraction(b[i, k, n])) for k in range(K))
                    assert abs(Fraction(c[i, m, n]) - exact) <= K * Fraction(2) ** -52 * max(exact_abs, Fraction(1, 10 ** 30))
                    assert abs(Fraction(s[i, m, n]) - exact_abs) <= K * Fraction(2) ** -52 * exact_abs


def test_selector_operand_copies_rows_of_the_other_operand():
    # A[b, k, m] = 1 where k == (2 m + b) mod K: C[b, m, :] = B[b, (2 m + b) mod K, :]. Reading A as
    # [M][K] instead of [K][M], or the wrong batch item, selects other rows.
    nb, M, N, K = 3, 5, 6, 11
    A = np.zeros((nb, K, M))
    for b in range(nb):
        for m in range(M):
            A[b, (2 * m + b) % K, m] = 1.0
    B = wl.normal_bf16(2, 1, (nb, K, N), 1.0)
    c, s = orc.batched_gemm_tn(bits(A), B)
    bv = vals(B)
    for b in range(nb):
        for m in range(M):
            assert np.array_equal(c[b, m], bv[b, (2 * m + b) % K])
            assert np.array_equal(s[b, m], np.abs(bv[b, (2 * m + b) % K]))


def test_integer_operands_give_exact_integers():
    nb, M, N, K = 2, 9, 7, 48
    A = wl.small_int_bf16(6, 0, (nb, K, M))
    B = wl.small_int_bf16(6, 1, (nb, K, N))
    c, s = orc.batched_gemm_tn(A, B)
    a, b = vals(A).astype(np.int64), vals(B).astype(np.int64)
    assert np.array_equal(c, np.einsum("bkm,bkn->bmn", a, b).astype(np.float64))
    assert np.array_equal(s, np.einsum("bkm,bkn->bmn", np.abs(a), np.abs(b)).astype(np.float64))


def test_one_item_is_a_matrix_product_of_the_transposed_operand():
    M, N, K = 13, 17, 150
    A = wl.normal_bf16(9, 0, (1, K, M), 1.0)
    B = wl.uniform_bf16(9, 1, (1, K, N), 0.1)
    c, _ = orc.batched_gemm_tn(A, B)
    want = vals(A)[0].T @ vals(B)[0]                 # library routine on the special case
    assert np.allclose(c[0], want, rtol=0, atol=K * 2.0 ** -50)


def test_scaling_and_batch_independence():
    nb, M, N, K = 3, 4, 5, 20
    A = wl.normal_bf16(14, 0, (nb, K, M), 1.0)
    B = wl.uniform_bf16(14, 1, (nb, K, N), 0.5)
    c, _ = orc.batched_gemm_tn(A, B)
    c2, _ = orc.batched_gemm_tn(A, bits(vals(B) * 0.25))
    assert np.array_equal(c2, 0.25 * c)
    A3 = A.copy()
    A3[1] = bits(-vals(A)[1])
    c3, _ = orc.batched_gemm_tn(A3, B)
    assert np.array_equal(c3[0], c[0]) and np.array_equal(c3[2], c[2]) and np.array_equal(c3[1], -c[1])


def test_empty_sizes_and_shape_errors():
    c, s = orc.batched_gemm_tn(np.zeros((2, 0, 3), np.uint16), np.zeros((2, 0, 4), np.uint16))
    assert c.shape == (2, 3, 4) and not c.any() and not s.any()
    with pytest.raises(ValueError):
        orc.batched_gemm_tn(np.zeros((2, 5, 3), np.uint16), np.zeros((2, 6, 4), np.uint16))


def test_generator_and_workload_figures():
    w = wl.BGEMM_WORKLOADS["T1"]
    A, B = wl.make_bgemm(w.batch, w.M, w.N, w.K, w.seed)
    A2, B2 = wl.make_bgemm(w.batch, w.M, w.N, w.K, w.seed)
    assert A.shape == (w.batch, w.K, w.M) and B.shape == (w.batch, w.K, w.N)
    assert np.array_equal(A, A2) and np.array_equal(B, B2)
    assert abs(vals(A).std() - 1.0) < 0.05 and np.abs(vals(B)).max() <= w.K ** -0.5 * (1 + 2.0 ** -8)
    assert w.flops == 2 * w.batch * w.M * w.N * w.K
    assert w.algorithmic_bytes == w.batch * (2 * w.K * (w.M + w.N) + 4 * w.M * w.N)
