"""The seeded input generator: determinism, chunk independence, distributions, bf16 rounding."""
import numpy as np

from paper_2512_09196_amd import workloads as wl


def test_splitmix64_first_outputs():
    # outputs of the published splitmix64 generator seeded with 0: the k-th output is
    # the finaliser applied to k * golden-gamma, i.e. _splitmix64((k-1) * gamma)
    gamma = 0x9E3779B97F4A7C15
    ctr = np.array([(k * gamma) & 0xFFFFFFFFFFFFFFFF for k in range(3)], dtype=np.uint64)
    got = wl._splitmix64(ctr)
    assert [int(x) for x in got] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


def test_deterministic_and_order_independent():
    a = wl.unit_uniform(3, 1, 0, 1000)
    b = np.concatenate([wl.unit_uniform(3, 1, 0, 400), wl.unit_uniform(3, 1, 400, 600)])
    assert np.array_equal(a, b)
    assert not np.array_equal(a, wl.unit_uniform(4, 1, 0, 1000))
    assert not np.array_equal(a, wl.unit_uniform(3, 2, 0, 1000))
    assert a.min() >= 0.0 and a.max() < 1.0


def test_bf16_rounding_nearest_even():
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -0.0, 3.0e38])
    bits = wl.f64_to_bf16_bits(x)
    assert list(bits[:5]) == [0x3F80, 0x3F80, 0x3F82, 0x3F81, 0x8000]
    back = wl.bf16_bits_to_f32(bits)
    assert back[0] == 1.0 and back[2] == 1.0 + 2.0 ** -6


def test_distributions_have_the_stated_moments():
    u = wl.bf16_bits_to_f32(wl.uniform_bf16(9, 0, (400, 500), 0.125)).astype(np.float64)
    assert abs(u.mean()) < 1e-3 and abs(u.std() - 0.125 / np.sqrt(3)) < 1e-3
    assert u.min() >= -0.125 and u.max() <= 0.125
    g = wl.bf16_bits_to_f32(wl.normal_bf16(9, 1, (400, 500), 0.02)).astype(np.float64)
    assert abs(g.mean()) < 2e-4 and abs(g.std() - 0.02) < 2e-4
    # kurtosis of a normal is 3: catches a broken Box-Muller
    assert abs(((g - g.mean()) ** 4).mean() / g.var() ** 2 - 3.0) < 0.1


def test_workload_table():
    w = wl.WORKLOADS
    assert [(w[k].M, w[k].N, w[k].K, w[k].seed) for k in ("C1", "C2", "C3", "C4", "C5")] == [
        (256, 256, 256, 0), (2048, 2048, 2048, 1), (4096, 11008, 4096, 2),
        (16, 8192, 8192, 3), (1024, 1024, 16384, 4)]
    assert w["C2"].flops == 2 * 2048 ** 3
    assert w["C4"].algorithmic_bytes == 2 * (16 * 8192 + 8192 * 8192 + 16 * 8192 + 8192)
    A, B, bias = wl.make_inputs(w["C1"])
    assert A.shape == (256, 256) and B.shape == (256, 256) and bias.shape == (256,)
    assert A.dtype == np.uint16
    assert np.abs(wl.bf16_bits_to_f32(A)).max() <= 1 / 16
