"""GPU parity of the batched vector-matrix product (the paper's Case Study 2,
C[m, n] = sum_k A[m, k] B[m, n, k]) against the CPU oracle, through the C ABI."""
import numpy as np
import pytest

from oracle import gemm_oracle as orc
from paper_2512_09196_amd import tf
from paper_2512_09196_amd import workloads as wl

import gpu_util as gu

pytestmark = pytest.mark.gpu


def bound(c, s, K):
    """Any-order fp32 accumulation of exact products: gamma_{K+1} s, doubled for the pairwise order of
    the lane exchange, plus half an ulp of the result."""
    return 2.0 * gu.gamma(K + 1) * s + 2.0 ** -23 * np.abs(c) + 1e-30


def strided3(bits, ld):
    out = np.full(bits.shape[:2] + (ld,), 0x7FC1, np.uint16)     # NaN patterns between the rows
    out[:, :, :bits.shape[2]] = bits
    return out


def check_all(M, N, K, A, B, lda=None, ldb=None, ldy=None, exact=False):
    c, s = orc.batched_vecmat(A, B)
    dA = gu.to_dev(A if lda is None else gu.strided(A, lda))
    dB = gu.to_dev(B if ldb is None else strided3(B, ldb))
    out = gu.OutBuf(M, N, ldy=ldy, f32=True)
    ran = []
    with tf.Problem(M, N, K, lda=lda, ldb=ldb, ldy=ldy, op=tf.TF_OP_BATCHED_VECMAT) as prob:
        for v in prob.variants():
            name = v.name.decode()
            print("case", (M, N, K), "variant", name, flush=True)
            got, intact, raw = gu.run_variant(prob, v.id, dA, dB, None, out)
            assert intact, "%s wrote outside C" % name
            assert not np.any(raw == gu.CANARY_F32), "%s left elements unwritten" % name
            if exact:
                assert np.array_equal(got, c), name
            else:
                err = np.abs(got - c)
                assert np.all(err <= bound(c, s, K)), "%s: worst excess %g" % (name, (err - bound(c, s, K)).max())
                assert np.all(err <= 1e-2 * (1.0 + np.abs(c))), name
            ran.append(name)
    return ran


def test_v1_every_variant():
    w = wl.VECMAT_WORKLOADS["V1"]
    A, B = wl.make_vecmat(w.M, w.N, w.K, w.seed)
    ran = check_all(w.M, w.N, w.K, A, B)
    assert ran[0] == "vecmat_naive_1elem_per_thread" and sum(n.startswith("vecmat_r") for n in ran) >= 3


@pytest.mark.parametrize("shape", [(3, 37, 520), (1, 1, 8), (5, 100, 4104), (2, 7, 512), (9, 1030, 64), (1, 3000, 2048)])
def test_ragged_rows_row_groups_and_k_chunks(shape):
    # N not a multiple of the rows per wave, K with a ragged last 512-chunk or shorter than one chunk,
    # more and fewer row groups than waves in the grid
    M, N, K = shape
    A, B = wl.make_vecmat(M, N, K, seed=100 + N)
    ran = check_all(M, N, K, A, B)
    assert any(n.startswith("vecmat_r") for n in ran)


@pytest.mark.parametrize("shape", [(4, 33, 1001), (2, 5, 3), (3, 10, 12)])
def test_k_not_a_multiple_of_eight_runs_on_the_naive_kernel_only(shape):
    M, N, K = shape
    A, B = wl.make_vecmat(M, N, K, seed=7 + K)
    ran = check_all(M, N, K, A, B)
    assert ran == ["vecmat_naive_1elem_per_thread"]


def test_leading_dimensions():
    M, N, K = 6, 75, 1032
    A, B = wl.make_vecmat(M, N, K, seed=55)
    check_all(M, N, K, A, B, lda=K + 8, ldb=K + 24, ldy=N + 5)


def test_integer_operands_are_bit_exact():
    M, N, K = 4, 130, 2048
    A = wl.small_int_bf16(9, 0, (M, K))
    B = wl.small_int_bf16(9, 1, (M, N, K))
    check_all(M, N, K, A, B, exact=True)


def test_degenerate_sizes_and_errors():
    torch = gu.torch_mod()
    # K = 0: C = 0
    out = gu.OutBuf(3, 5, f32=True)
    with tf.Problem(3, 5, 0, op=tf.TF_OP_BATCHED_VECMAT) as prob:
        assert [v.name.decode() for v in prob.variants()] == ["vecmat_naive_1elem_per_thread"]
        got, intact, _ = gu.run_variant(prob, 0, None, None, None, out)
        assert intact and not got.any()
    # M = 0 or N = 0: nothing is launched
    with tf.Problem(0, 5, 8, op=tf.TF_OP_BATCHED_VECMAT) as prob:
        prob.run(0, None, None, None, None)
    # the output must be fp32, the rows of B at least K long
    with pytest.raises(tf.TfError):
        tf.Problem(2, 2, 16, ldb=8, op=tf.TF_OP_BATCHED_VECMAT)
    A, B = wl.make_vecmat(2, 16, 64, seed=1)
    dA, dB = gu.to_dev(A), gu.to_dev(B)
    out = gu.OutBuf(2, 16, f32=True)
    with tf.Problem(2, 16, 64, op=tf.TF_OP_BATCHED_VECMAT) as prob:
        stream_v = [v for v in prob.variants() if v.kind == tf.TF_KIND_VECMAT_STREAM][0]
        with pytest.raises(tf.TfError) as e:
            prob.run(stream_v.id, dA.data_ptr() + 2, dB, None, out.ptr)      # misaligned A
        assert e.value.status == tf.TF_E_UNSUPPORTED
    torch.cuda.synchronize()


def test_variant_loop_on_v1():
    torch = gu.torch_mod()
    w = wl.VECMAT_WORKLOADS["V1"]
    A, B = wl.make_vecmat(w.M, w.N, w.K, w.seed)
    c, s = orc.batched_vecmat(A, B)
    dA, dB = gu.to_dev(A), gu.to_dev(B)
    Y = torch.empty((w.M, w.N), dtype=torch.float32, device="cuda")
    with tf.Problem(w.M, w.N, w.K, op=tf.TF_OP_BATCHED_VECMAT) as prob:
        best, rep, log = prob.tune(dA, dB, None, Y)
        print("V1 tune ->", prob.variants()[best].name.decode(), "%.2f us" % rep.t_med_us, "rounds", len(log) - 1, flush=True)
        assert log[0].variant_id == 0 and 1 <= len(log) - 1 <= 8
        assert rep.parity_ok == 1 and rep.status == 0
        got = Y.double().cpu().numpy()
        assert np.all(np.abs(got - c) <= bound(c, s, w.K))


def test_full_size_v2_against_the_whole_oracle():
    torch = gu.torch_mod()
    w = wl.VECMAT_WORKLOADS["V2"]
    A, B = wl.make_vecmat(w.M, w.N, w.K, w.seed)
    c, s = orc.batched_vecmat(A, B)
    dA, dB = gu.to_dev(A), gu.to_dev(B)
    del B
    Y = torch.empty((w.M, w.N), dtype=torch.float32, device="cuda")
    with tf.Problem(w.M, w.N, w.K, op=tf.TF_OP_BATCHED_VECMAT) as prob:
        for v in prob.variants():
            if v.kind == tf.TF_KIND_VECMAT_NAIVE:
                continue
            print("V2", v.name.decode(), flush=True)
            Y.fill_(float("nan"))
            prob.run(v.id, dA, dB, None, Y)
            got = Y.double().cpu().numpy()
            assert not np.isnan(got).any(), v.name.decode()
            assert np.all(np.abs(got - c) <= bound(c, s, w.K)), v.name.decode()
        best, rep, log = prob.tune(dA, dB, None, Y)
        name = prob.variants()[best].name.decode()
        print("V2 tune ->", name, "%.2f us" % rep.t_med_us, "%.0f GB/s" % rep.gbytes_per_s, "rounds", len(log) - 1, flush=True)
        assert best != 0 and log[0].t_med_us / rep.t_med_us >= 1.05
        got = Y.double().cpu().numpy()
        assert np.all(np.abs(got - c) <= bound(c, s, w.K))
