"""Pins for the CPU oracle of  Y = GELU_erf(A.B + bias).

None of the expected values below is produced by the oracle: they come from
exact rational arithmetic, from a power series evaluated in high-precision
decimals, from normal-table constants, from algebraic identities and from
numpy's own float64 matmul.  Each test is chosen to fail on one plausible
mistake (dropped bias, wrong sign in erf, transposed operand, wrong stride,
tanh-GELU instead of erf-GELU, fp32 instead of double accumulation ...).
"""
import math
from decimal import Decimal, getcontext
from fractions import Fraction

import numpy as np
import pytest

from oracle import gemm_oracle as orc
from paper_2512_09196_amd import workloads as wl


# ----------------------------------------------------------------- helpers
def bf16_fraction(bits: int) -> Fraction:
    """Exact rational value of a (finite) bf16 bit pattern, decoded field by field."""
    sign = -1 if bits & 0x8000 else 1
    e = (bits >> 7) & 0xFF
    m = bits & 0x7F
    assert e != 0xFF
    if e == 0:
        return sign * Fraction(m, 1 << 7) * Fraction(1, 1 << 126)
    return sign * (1 + Fraction(m, 1 << 7)) * (Fraction(2) ** (e - 127))


def phi_decimal(x: float) -> Decimal:
    """Standard normal CDF from the Maclaurin series of erf, in 80-digit decimals."""
    getcontext().prec = 80
    t = Decimal(x) / Decimal(2).sqrt()
    term = t
    total = t
    n = 0
    while abs(term) > Decimal(10) ** -70:
        n += 1
        term = -term * t * t / n
        total += term / (2 * n + 1)
    pi = Decimal("3.14159265358979323846264338327950288419716939937510582097494459230781640628620899")
    erf = 2 * total / pi.sqrt()
    return (1 + erf) / 2


# ----------------------------------------------------------------- bf16 decode
def test_bf16_decode_matches_field_decode():
    rng = np.random.default_rng(7)
    pats = list(rng.integers(0, 1 << 16, 400)) + [0, 0x8000, 1, 0x7F, 0x80, 0x3F80, 0xBF80, 0x7F7F, 0xFF7F]
    for b in pats:
        b = int(b)
        if (b >> 7) & 0xFF == 0xFF:
            continue
        assert Fraction(orc.bf16_to_double(b)) == bf16_fraction(b)
    assert orc.bf16_to_double(0x3F80) == 1.0
    assert orc.bf16_to_double(0xC000) == -2.0
    assert math.isinf(orc.bf16_to_double(0x7F80))
    assert math.isnan(orc.bf16_to_double(0x7FC0))


# ----------------------------------------------------------------- GELU scalar
def test_gelu_zero_is_zero():
    assert orc.gelu(0.0) == 0.0


# x, Phi(x) to the nine digits any normal table prints.
_NORMAL_TABLE = [(0.5, 0.691462461), (1.0, 0.841344746), (1.5, 0.933192799),
                 (2.0, 0.977249868), (2.5, 0.993790335), (3.0, 0.998650102)]


@pytest.mark.parametrize("x,phi", _NORMAL_TABLE)
def test_gelu_against_normal_table(x, phi):
    assert orc.gelu(x) == pytest.approx(x * phi, abs=2e-9)
    assert orc.gelu(-x) == pytest.approx(-x * (1.0 - phi), abs=2e-9)


@pytest.mark.parametrize("x", [-8.0, -6.0, -3.0, -2.0, -1.0, -0.75179, -0.5, -1e-3, 1e-3,
                               0.5, 1.0, math.sqrt(2.0), 2.0, 3.0, 6.0, 8.0])
def test_gelu_against_decimal_series(x):
    want = Decimal(x) * phi_decimal(x)
    got = orc.gelu(x)
    # relative accuracy also in the negative tail, where 1 + erf cancels; the tail is
    # ill conditioned (d ln erfc(t) / d ln t ~ 2 t^2), so rounding x / sqrt 2 alone costs x^2 ulp
    assert abs(Decimal(got) - want) <= abs(want) * Decimal((4 + x * x) * 2.2e-16) + Decimal("1e-300")


def test_gelu_odd_part_identity():
    # Phi(x) + Phi(-x) = 1  =>  GELU(x) - GELU(-x) = x
    for x in np.linspace(-9, 9, 361):
        assert orc.gelu(x) - orc.gelu(-x) == pytest.approx(x, abs=4e-15 * max(1, abs(x)))


def test_gelu_is_erf_form_not_tanh_form():
    # the tanh approximation differs from x*Phi(x) by ~1e-4 at |x| = 2
    x = 2.0
    tanh_form = 0.5 * x * (1 + math.tanh(math.sqrt(2 / math.pi) * (x + 0.044715 * x ** 3)))
    assert abs(orc.gelu(x) - tanh_form) > 5e-5
    assert abs(orc.gelu(x) - float(Decimal(x) * phi_decimal(x))) < 1e-14


def gelu_tanh_decimal(x: float) -> Decimal:
    """1/2 x (1 + tanh u) with tanh u = (e^{2u} - 1) / (e^{2u} + 1), 50 digits; sqrt(2/pi) from a 50-digit pi."""
    getcontext().prec = 60
    pi = Decimal("3.14159265358979323846264338327950288419716939937510")
    xd = Decimal(x)
    u = (Decimal(2) / pi).sqrt() * (xd + Decimal("0.044715") * xd ** 3)
    e = (2 * u).exp()
    return xd / 2 * (1 + (e - 1) / (e + 1))


@pytest.mark.parametrize("x", [-9.0, -5.0, -3.0, -1.5, -0.75, -1e-3, 1e-6, 0.3, 1.0, 2.0, 3.5, 6.0, 12.0])
def test_gelu_tanh_against_decimal_evaluation(x):
    want = gelu_tanh_decimal(x)
    got = orc.gelu_tanh(x)
    # 1 + tanh cancels on the negative side: allow the absolute error of tanh (one ulp of 1) times |x| / 2
    assert abs(Decimal(got) - want) <= abs(want) * Decimal(1e-15) + Decimal(abs(x) * 1.2e-16)


def test_gelu_tanh_identities_limits_and_distance_from_the_erf_form():
    xs = np.linspace(-9, 9, 361)
    y = orc.gelu_tanh(xs)
    # tanh is odd: GELU_tanh(x) - GELU_tanh(-x) = x
    assert np.allclose(y - orc.gelu_tanh(-xs), xs, rtol=0, atol=4e-15 * 9)
    assert orc.gelu_tanh(0.0) == 0.0 and orc.gelu_tanh(40.0) == 40.0 and abs(orc.gelu_tanh(-40.0)) == 0.0
    assert np.array_equal(y, np.array([orc.gelu_tanh(float(x)) for x in xs]))      # array and scalar entry agree
    # an approximation of x Phi(x): within 5e-4 everywhere, and not equal to it
    d = np.abs(y - np.array([orc.gelu(float(x)) for x in xs]))
    assert d.max() < 5e-4 and d.max() > 1e-4
    # slope 1/2 at the origin
    h = 1e-6
    assert (orc.gelu_tanh(h) - orc.gelu_tanh(-h)) / (2 * h) == pytest.approx(0.5, abs=1e-9)


def test_gelu_minimum_and_limits():
    xs = np.linspace(-2, 0, 20001)
    ys = np.array([orc.gelu(x) for x in xs])
    i = int(np.argmin(ys))
    assert xs[i] == pytest.approx(-0.75179, abs=2e-4)
    assert ys[i] == pytest.approx(-0.169971207, abs=1e-8)
    assert orc.gelu(40.0) == 40.0
    assert orc.gelu(-40.0) == 0.0 or abs(orc.gelu(-40.0)) < 1e-300


# ----------------------------------------------------------------- GEMM: exact brute force
@pytest.mark.parametrize("shape", [(1, 1, 1), (2, 3, 4), (5, 1, 7), (1, 6, 2), (7, 5, 3), (17, 19, 23)])
def test_gemm_exact_rational_bruteforce(shape):
    M, N, K = shape
    A, B, bias = wl.make_custom(M, N, K, seed=100 + M + N + K,
                                a_dist=("normal", 1.0), b_dist=("normal", 0.5))
    y, z, s = orc.gemm_bias_gelu(A, B, bias)
    for m in range(M):
        for n in range(N):
            acc = Fraction(0)
            sabs = Fraction(0)
            for k in range(K):
                p = bf16_fraction(int(A[m, k])) * bf16_fraction(int(B[k, n]))
                acc += p
                sabs += abs(p)
            bv = bf16_fraction(int(bias[n]))
            zz = acc + bv
            ss = sabs + abs(bv)
            assert abs(Fraction(z[m, n]) - zz) <= Fraction(K + 1, 1 << 52) * ss
            assert abs(Fraction(s[m, n]) - ss) <= Fraction(K + 1, 1 << 52) * ss
            want_y = float(Decimal(float(zz)) * phi_decimal(float(zz)))
            assert y[m, n] == pytest.approx(want_y, rel=1e-13, abs=1e-15 * float(ss))


def test_gemm_against_numpy_float64_matmul():
    # non-square, asymmetric distributions: a transposed operand or swapped stride fails
    M, N, K = 37, 53, 129
    A, B, bias = wl.make_custom(M, N, K, seed=5, a_dist=("normal", 1.0), b_dist=("uniform", 0.25))
    Af = wl.bf16_bits_to_f32(A).astype(np.float64)
    Bf = wl.bf16_bits_to_f32(B).astype(np.float64)
    bf = wl.bf16_bits_to_f32(bias).astype(np.float64)
    y, z, s = orc.gemm_bias_gelu(A, B, bias)
    zz = Af @ Bf + bf[None, :]
    ss = np.abs(Af) @ np.abs(Bf) + np.abs(bf)[None, :]
    assert np.all(np.abs(z - zz) <= 1e-13 * ss)
    assert np.all(np.abs(s - ss) <= 1e-13 * ss)
    from scipy.special import ndtr
    assert np.allclose(y, zz * ndtr(zz), rtol=1e-12, atol=1e-14)


def test_gemm_sampled_entry_equals_full_entry():
    M, N, K = 23, 41, 77
    A, B, bias = wl.make_custom(M, N, K, seed=11)
    y, z, s = orc.gemm_bias_gelu(A, B, bias)
    rows = np.array([0, 22, 5, 13, 22], np.int32)
    cols = np.array([0, 40, 17, 2, 0], np.int32)
    y2, z2, s2 = orc.gemm_bias_gelu_at(A, B, bias, rows, cols)
    # same sum in the same order (increasing k): identical doubles
    assert np.array_equal(z2, z[rows, cols])
    assert np.array_equal(y2, y[rows, cols])
    assert np.array_equal(s2, s[rows, cols])
    # and pinned on its own against the exact rational value
    for t in range(len(rows)):
        acc = sum(bf16_fraction(int(A[rows[t], k])) * bf16_fraction(int(B[k, cols[t]])) for k in range(K))
        acc += bf16_fraction(int(bias[cols[t]]))
        assert abs(Fraction(z2[t]) - acc) <= Fraction(K + 1, 1 << 52) * Fraction(s2[t])


# ----------------------------------------------------------------- GEMM: structured operands
def _bits(x):
    return wl.f64_to_bf16_bits(np.asarray(x, np.float64))


def test_identity_A_gives_gelu_of_B_plus_bias():
    K, N = 24, 31
    _, B, bias = wl.make_custom(K, N, K, seed=3, b_dist=("normal", 1.0))
    A = _bits(np.eye(K))
    y, z, s = orc.gemm_bias_gelu(A, B, bias)
    want_z = wl.bf16_bits_to_f32(B).astype(np.float64) + wl.bf16_bits_to_f32(bias).astype(np.float64)[None, :]
    assert np.array_equal(z, want_z)
    from scipy.special import ndtr
    assert np.allclose(y, want_z * ndtr(want_z), rtol=1e-12, atol=1e-15)


def test_zero_A_gives_gelu_of_bias_and_all_zero_gives_zero():
    M, N, K = 9, 14, 33
    _, B, bias = wl.make_custom(M, N, K, seed=4)
    A = np.zeros((M, K), np.uint16)
    y, z, s = orc.gemm_bias_gelu(A, B, bias)
    bf = wl.bf16_bits_to_f32(bias).astype(np.float64)
    assert np.array_equal(z, np.broadcast_to(bf, (M, N)))
    assert np.array_equal(s, np.broadcast_to(np.abs(bf), (M, N)))
    y0, z0, s0 = orc.gemm_bias_gelu(A, B, np.zeros(N, np.uint16))
    assert np.all(y0 == 0.0) and np.all(z0 == 0.0) and np.all(s0 == 0.0)


def test_ones_A_gives_column_sums():
    M, N, K = 6, 10, 64
    _, B, bias = wl.make_custom(M, N, K, seed=8, b_dist=("normal", 1.0))
    A = _bits(np.ones((M, K)))
    y, z, s = orc.gemm_bias_gelu(A, B, bias)
    Bf = wl.bf16_bits_to_f32(B).astype(np.float64)
    want = np.array([math.fsum(Bf[:, n]) for n in range(N)]) + wl.bf16_bits_to_f32(bias).astype(np.float64)
    assert np.allclose(z, np.broadcast_to(want, (M, N)), rtol=0, atol=1e-13)
    assert np.all(y == y[0:1, :])


def test_rank_one_closed_form():
    M, N, K = 8, 12, 16
    u = np.arange(1, M + 1, dtype=np.float64) * 0.25          # exact in bf16
    v = np.arange(-6, N - 6, dtype=np.float64) * 0.5
    A = _bits(np.outer(u, np.ones(K)) / K)                     # K = 16: exact scaling
    B = _bits(np.outer(np.ones(K), v))
    bias = np.zeros(N, np.uint16)
    _, z, _ = orc.gemm_bias_gelu(A, B, bias)
    assert np.array_equal(z, np.outer(u, v))


def test_power_of_two_scaling_is_exact():
    M, N, K = 11, 13, 57
    A, B, _ = wl.make_custom(M, N, K, seed=21)
    zero = np.zeros(N, np.uint16)
    _, z1, _ = orc.gemm_bias_gelu(A, B, zero)
    A2 = (A + np.uint16(1 << 7)).astype(np.uint16)            # exponent + 1 : exactly 2*A
    assert np.array_equal(wl.bf16_bits_to_f32(A2), 2 * wl.bf16_bits_to_f32(A))
    _, z2, _ = orc.gemm_bias_gelu(A2, B, zero)
    assert np.array_equal(z2, 2.0 * z1)


def test_k_permutation_invariance():
    M, N, K = 7, 9, 101
    A, B, bias = wl.make_custom(M, N, K, seed=22)
    perm = np.random.default_rng(0).permutation(K)
    _, z1, s1 = orc.gemm_bias_gelu(A, B, bias)
    _, z2, s2 = orc.gemm_bias_gelu(A[:, perm].copy(), B[perm, :].copy(), bias)
    assert np.all(np.abs(z1 - z2) <= (K + 1) * 2.0 ** -52 * s1)


def test_integer_operands_are_exact():
    M, N, K = 19, 21, 300
    A = wl.small_int_bf16(31, 0, (M, K))
    B = wl.small_int_bf16(31, 1, (K, N))
    bias = wl.small_int_bf16(31, 2, (N,), -3, 3)
    _, z, _ = orc.gemm_bias_gelu(A, B, bias)
    Ai = wl.bf16_bits_to_f32(A).astype(np.int64)
    Bi = wl.bf16_bits_to_f32(B).astype(np.int64)
    bi = wl.bf16_bits_to_f32(bias).astype(np.int64)
    assert set(np.unique(Ai)) <= {-2, -1, 0, 1, 2} and len(np.unique(Ai)) == 5
    assert np.array_equal(z, (Ai @ Bi + bi[None, :]).astype(np.float64))


def test_double_accumulation_not_float():
    # 1 + 2^-30 * 2^12 terms: lost entirely by an fp32 accumulator, kept by double
    K = 4096
    A = _bits(np.concatenate([[1.0], np.full(K - 1, 2.0 ** -15)]))[None, :]
    B = _bits(np.concatenate([[1.0], np.full(K - 1, 2.0 ** -15)]))[:, None]
    _, z, _ = orc.gemm_bias_gelu(A, B, np.zeros(1, np.uint16))
    assert z[0, 0] == 1.0 + (K - 1) * 2.0 ** -30


def test_empty_shapes():
    y, z, s = orc.gemm_bias_gelu(np.zeros((0, 5), np.uint16), np.zeros((5, 4), np.uint16), np.zeros(4, np.uint16))
    assert y.shape == (0, 4)
    bias = _bits(np.array([0.5, -1.0, 2.0]))
    y, z, s = orc.gemm_bias_gelu(np.zeros((2, 0), np.uint16), np.zeros((0, 3), np.uint16), bias)
    assert np.array_equal(z, np.broadcast_to(np.array([0.5, -1.0, 2.0]), (2, 3)))


def test_bad_arguments_are_rejected():
    with pytest.raises(TypeError):
        orc.gemm_bias_gelu(np.zeros((2, 2), np.float32), np.zeros((2, 2), np.uint16), np.zeros(2, np.uint16))
    with pytest.raises(ValueError):
        orc.gemm_bias_gelu(np.zeros((2, 3), np.uint16), np.zeros((2, 2), np.uint16), np.zeros(2, np.uint16))
    with pytest.raises(RuntimeError):
        orc.gemm_bias_gelu_at(np.zeros((2, 2), np.uint16), np.zeros((2, 2), np.uint16), np.zeros(2, np.uint16),
                              [2], [0])
