"""Pins for the oracle of the tile kernel with the second operand given as [N][K]
(z[m, n] = sum_k a[m, k] bt[n, k] + bias[n], y = GELU_erf(z)). None of the expected values comes
from the oracle function under test."""
from fractions import Fraction
import math

import numpy as np

from oracle import gemm_oracle as orc
from paper_2512_09196_amd import workloads as wl


def bits(x):
    return wl.f64_to_bf16_bits(np.asarray(x, dtype=np.float64))


def vals(b):
    return wl.bf16_bits_to_f32(b).astype(np.float64)


def phi(x):
    return 0.5 * math.erfc(-x / math.sqrt(2.0))      # the normal CDF, from the standard library


def test_exact_rational_brute_force_on_small_cases():
    rng = np.random.default_rng(21)
    for (M, N, K) in ((1, 1, 1), (3, 4, 5), (5, 2, 9), (2, 7, 23)):
        A = bits(rng.normal(0, 1, (M, K)))
        Bt = bits(rng.uniform(-1, 1, (N, K)))
        bias = bits(rng.normal(0, 1, N))
        y, z, s = orc.gemm_nt_bias_gelu(A, Bt, bias)
        a, b, c = vals(A), vals(Bt), vals(bias)
        for m in range(M):
            for n in range(N):
                exact = sum(Fraction(a[m, k]) * Fraction(b[n, k]) for k in range(K)) + Fraction(c[n])
                exact_abs = sum(abs(Fraction(a[m, k]) * Fraction(b[n, k])) for k in range(K)) + abs(Fraction(c[n]))
                assert abs(Fraction(z[m, n]) - exact) <= (K + 1) * Fraction(2) ** -52 * exact_abs
                assert abs(Fraction(s[m, n]) - exact_abs) <= (K + 1) * Fraction(2) ** -52 * exact_abs
                zf = float(exact)
                assert abs(y[m, n] - zf * phi(zf)) <= 4e-16 * (1 + abs(zf))


def test_selector_operand_copies_columns_of_a():
    # bt[n, k] = 1 where k == (3 n + 1) mod K: z[:, n] = a[:, (3 n + 1) mod K] + bias[n]. Reading Bt as [K][N]
    # instead of [N][K] (or with the wrong leading dimension) selects other columns.
    M, N, K = 6, 5, 11
    Bt = np.zeros((N, K))
    for n in range(N):
        Bt[n, (3 * n + 1) % K] = 1.0
    A = wl.normal_bf16(3, 0, (M, K), 1.0)
    bias = wl.normal_bf16(3, 2, (N,), 1.0)
    y, z, s = orc.gemm_nt_bias_gelu(A, bits(Bt), bias)
    a, c = vals(A), vals(bias)
    for n in range(N):
        col = a[:, (3 * n + 1) % K]
        assert np.array_equal(z[:, n], col + c[n])
        assert np.array_equal(s[:, n], np.abs(col) + abs(c[n]))


def test_integer_operands_give_exact_integers():
    M, N, K = 9, 7, 64
    A = wl.small_int_bf16(8, 0, (M, K))
    Bt = wl.small_int_bf16(8, 1, (N, K))
    bias = wl.small_int_bf16(8, 2, (N,), -3, 3)
    y, z, s = orc.gemm_nt_bias_gelu(A, Bt, bias)
    a, b, c = vals(A).astype(np.int64), vals(Bt).astype(np.int64), vals(bias).astype(np.int64)
    assert np.array_equal(z, (np.einsum("mk,nk->mn", a, b) + c[None, :]).astype(np.float64))
    assert np.array_equal(s, (np.einsum("mk,nk->mn", np.abs(a), np.abs(b)) + np.abs(c)[None, :]).astype(np.float64))


def test_library_product_of_the_explicitly_transposed_operand():
    M, N, K = 13, 17, 150
    A = wl.normal_bf16(9, 0, (M, K), 1.0)
    Bt = wl.uniform_bf16(9, 1, (N, K), 0.1)
    bias = wl.normal_bf16(9, 2, (N,), 0.5)
    y, z, s = orc.gemm_nt_bias_gelu(A, Bt, bias)
    want = vals(A) @ vals(Bt).T + vals(bias)[None, :]        # library routine on the same numbers
    assert np.allclose(z, want, rtol=0, atol=K * 2.0 ** -48)
    # a non-square operand read with rows and columns swapped gives something else entirely
    wrong = vals(A) @ vals(Bt).reshape(K, N) + vals(bias)[None, :]
    assert np.abs(z - wrong).max() > 1e-3


def test_scaling_zero_matrix_and_gelu_of_zero():
    M, N, K = 4, 6, 20
    A = wl.normal_bf16(14, 0, (M, K), 1.0)
    Bt = wl.uniform_bf16(14, 1, (N, K), 0.5)
    zero_bias = np.zeros(N, np.uint16)
    _, z, _ = orc.gemm_nt_bias_gelu(A, Bt, zero_bias)
    _, z2, _ = orc.gemm_nt_bias_gelu(A, bits(vals(Bt) * 0.25), zero_bias)
    assert np.array_equal(z2, 0.25 * z)                      # power-of-two scaling is exact
    bias = wl.normal_bf16(14, 2, (N,), 1.0)
    y, z, s = orc.gemm_nt_bias_gelu(np.zeros((M, K), np.uint16), Bt, bias)
    c = vals(bias)
    assert np.array_equal(z, np.broadcast_to(c, (M, N)))
    assert np.allclose(y, np.broadcast_to([v * phi(v) for v in c], (M, N)), rtol=0, atol=3e-16)
    y0, z0, s0 = orc.gemm_nt_bias_gelu(np.zeros((M, K), np.uint16), np.zeros((N, K), np.uint16), zero_bias)
    assert not y0.any() and not z0.any() and not s0.any()    # GELU(0) = 0
    # K = 0: the sum is empty
    y1, z1, _ = orc.gemm_nt_bias_gelu(np.zeros((M, 0), np.uint16), np.zeros((N, 0), np.uint16), bias)
    assert np.array_equal(z1, np.broadcast_to(c, (M, N)))
