"""Pins for the element-wise sine oracle (the paper's Case Study 1). No expected value comes from the oracle."""
from fractions import Fraction
import math

import numpy as np
import pytest

from oracle import gemm_oracle as orc
from paper_2512_09196_amd import workloads as wl


def taylor_sin(x: Fraction, terms: int = 40) -> Fraction:
    """sin x as an exact rational partial sum; for |x| <= 6 the remainder after 40 terms is below 1e-60."""
    s, term = Fraction(0), x
    for k in range(terms):
        s += term
        term = -term * x * x / ((2 * k + 2) * (2 * k + 3))
    return s


def test_exact_rational_taylor_sums_of_the_binary32_inputs():
    rng = np.random.default_rng(4)
    x = np.concatenate([rng.uniform(-6, 6, 60), [0.5, 1.0, 3.0, -2.5, 1e-3, -1e-6]]).astype(np.float32)
    y = orc.sin_f32(x)
    for xi, yi in zip(x, y):
        want = taylor_sin(Fraction(float(xi)))
        assert abs(Fraction(float(yi)) - want) <= Fraction(2) ** -52, (xi, yi)     # libm sin: below one ulp of double


def test_symmetry_zeros_and_range():
    x = wl.make_sin_input(5000, seed=3, sigma=50.0)
    y = orc.sin_f32(x)
    assert np.array_equal(orc.sin_f32(-x), -y)
    assert np.all(np.abs(y) <= 1.0)
    z = orc.sin_f32(np.array([0.0, -0.0], np.float32))
    assert z[0] == 0.0 and z[1] == 0.0 and math.copysign(1.0, z[1]) == -1.0


def test_near_multiples_of_pi():
    # x = fl32(k pi): sin x = (-1)^k (x - k pi) (1 - O((x - k pi)^2)), with k pi taken from a 60-digit constant
    PI = Fraction(3141592653589793238462643383279502884197169399375105820974944, 10 ** 60)
    ks = np.array([1, 2, 3, 7, 10, 22, 100, 355], np.int64)
    x = (ks * math.pi).astype(np.float32)
    y = orc.sin_f32(x)
    for k, xi, yi in zip(ks, x, y):
        d = Fraction(float(xi)) - int(k) * PI
        want = (-1) ** int(k) * (d - d ** 3 / 6)
        assert abs(Fraction(float(yi)) - want) <= abs(want) * Fraction(1, 10 ** 12) + Fraction(1, 10 ** 25)


def test_generator_and_workload_figures():
    w = wl.SIN_WORKLOADS["E1"]
    x = wl.make_sin_input(w.n, w.seed)
    assert x.dtype == np.float32 and x.shape == (w.n,) and np.array_equal(x, wl.make_sin_input(w.n, w.seed))
    assert abs(x.mean()) < 0.2 and abs(x.std() - 10.0) < 0.2
    assert w.algorithmic_bytes == 8 * w.n and w.flops == w.n
    with pytest.raises(ValueError):
        orc.sin_f32(np.zeros(4, np.float64))
