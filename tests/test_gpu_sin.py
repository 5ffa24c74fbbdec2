"""GPU parity of the element-wise sine (the paper's Case Study 1, y[i] = sin(x[i]) at many launch shapes)
against the CPU oracle, through the C ABI."""
import numpy as np
import pytest

from oracle import gemm_oracle as orc
from paper_2512_09196_amd import tf
from paper_2512_09196_amd import workloads as wl

import gpu_util as gu

pytestmark = pytest.mark.gpu

# |x| <= 1e4: the quotient by pi/2 has at most 13 bits, so the first reduction step is exact and the two
# that follow round once each (2 * 2^-25 on |r| < 1); the polynomials add under 2^-26, the last
# rounding 2^-25: below 2^-23 in all. The bar leaves a factor of two.
TOL = 2.0 ** -22


def check_all(x, offset=0):
    """Every variant on x placed `offset` floats into 16-byte aligned buffers. Returns the names that ran."""
    torch = gu.torch_mod()
    n = x.shape[0]
    want = orc.sin_f32(x)
    guard = 64
    dx = torch.zeros(n + offset + 4, dtype=torch.float32, device="cuda")
    dx[offset:offset + n] = torch.from_numpy(x).cuda()
    dy = torch.empty(guard + offset + n + guard, dtype=torch.float32, device="cuda")
    xp = dx.data_ptr() + 4 * offset
    yp = dy.data_ptr() + 4 * (guard + offset)
    ran, first = [], None
    with tf.Problem(1, n, 0, op=tf.TF_OP_ELEMENTWISE_SIN) as prob:
        for v in prob.variants():
            name = v.name.decode()
            print("n", n, "offset", offset, "variant", name, flush=True)
            dy.fill_(float(gu.CANARY_F32))
            if offset % 4 and v.bk > 1 and (4 * offset) % (4 * v.bk):
                with pytest.raises(tf.TfError):
                    prob.run(v.id, xp, None, None, yp)
                continue
            prob.run(v.id, xp, None, None, yp)
            torch.cuda.synchronize()
            h = dy.cpu().numpy()
            body = h[guard + offset:guard + offset + n]
            assert np.all(h[:guard + offset] == gu.CANARY_F32) and np.all(h[guard + offset + n:] == gu.CANARY_F32), \
                "%s wrote outside y" % name
            assert not np.any(body == gu.CANARY_F32), "%s left elements unwritten" % name
            err = np.abs(body.astype(np.float64) - want)
            assert np.all(err <= TOL), "%s: worst error %g at x = %r" % (name, err.max(), x[err.argmax()])
            if first is None:
                first = body.copy()
            else:
                assert np.array_equal(first.view(np.uint32), body.view(np.uint32)), name   # one arithmetic, many shapes
            ran.append(name)
    return ran


def test_e1_every_variant():
    w = wl.SIN_WORKLOADS["E1"]
    ran = check_all(wl.make_sin_input(w.n, w.seed))
    assert ran[0] == "sin_block4_t64" and len(ran) >= 10


@pytest.mark.parametrize("n", [1, 3, 4, 5, 63, 64, 255, 1023, 4097, 16384, 70001])
def test_ragged_lengths(n):
    check_all(wl.make_sin_input(n, seed=40 + n % 7))


def test_large_arguments_special_values_and_signs():
    x = np.clip(wl.make_sin_input(50000, seed=41, sigma=1000.0), -1e4, 1e4)
    k = np.arange(1, 3001)
    x = np.concatenate([x, (k * np.pi).astype(np.float32), (-(k - 0.5) * np.pi).astype(np.float32),
                        np.array([0.0, -0.0, 1e-30, -1e-30, 1e-8, np.pi / 4, -np.pi / 4, 1e4, -1e4], np.float32)])
    check_all(x.astype(np.float32))
    torch = gu.torch_mod()
    z = torch.tensor([0.0, -0.0, float("nan")], dtype=torch.float32, device="cuda")
    y = torch.empty(3, dtype=torch.float32, device="cuda")
    with tf.Problem(1, 3, 0, op=tf.TF_OP_ELEMENTWISE_SIN) as prob:
        for v in prob.variants():
            prob.run(v.id, z, None, None, y)
            h = y.cpu().numpy()
            assert h[0] == 0 and h[1] == 0 and np.signbit(h[1]) and not np.signbit(h[0]) and np.isnan(h[2])


def test_misaligned_buffers():
    # the vector variants refuse pointers that are not aligned to their access width; the scalar ones run
    x = wl.make_sin_input(5001, seed=42)
    ran1 = check_all(x, offset=1)
    ran2 = check_all(x, offset=2)
    assert all("_v1_" in n or n == "sin_block4_t64" for n in ran1) and len(ran1) >= 3
    assert any("_v2_" in n for n in ran2) and not any("_v4_" in n for n in ran2)


def test_empty_input_is_a_no_op():
    torch = gu.torch_mod()
    y = torch.full((8,), 7.0, dtype=torch.float32, device="cuda")
    with tf.Problem(1, 0, 0, op=tf.TF_OP_ELEMENTWISE_SIN) as prob:
        for v in prob.variants():
            prob.run(v.id, y, None, None, y)
    torch.cuda.synchronize()
    assert bool((y == 7.0).all().item())


@pytest.mark.parametrize("name", ["E1", "E2"])
def test_tune(name):
    torch = gu.torch_mod()
    w = wl.SIN_WORKLOADS[name]
    x = wl.make_sin_input(w.n, w.seed)
    dx = torch.from_numpy(x).cuda()
    dy = torch.empty(w.n, dtype=torch.float32, device="cuda")
    with tf.Problem(1, w.n, 0, op=tf.TF_OP_ELEMENTWISE_SIN) as prob:
        best, rep, log = prob.tune(dx, None, None, dy)
        vs = prob.variants()
        print(name, "tune ->", vs[best].name.decode(), "%.2f us" % rep.t_med_us, "%.0f GB/s" % rep.gbytes_per_s,
              "baseline %.2f us" % log[0].t_med_us, flush=True)
        assert log[0].variant_id == 0 and best != 0 and rep.parity_ok == 1 and rep.status == 0
        assert all(r.parity_ok == 1 for r in log if r.status == 0)
        assert log[0].t_med_us / rep.t_med_us >= (20.0 if name == "E2" else 1.05)
    # sampled against the oracle at the full size
    idx = np.unique(np.concatenate([np.arange(0, 4096), np.arange(w.n - 4096, w.n),
                                    np.random.default_rng(5).integers(0, w.n, 200000)]))
    got = dy[torch.from_numpy(idx).cuda()].cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - orc.sin_f32(x[idx])) <= TOL)
