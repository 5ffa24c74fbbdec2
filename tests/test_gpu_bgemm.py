"""GPU parity of the batched transposed-operand product (the paper's Case Study 3,
C[b, m, n] = sum_k A[b, k, m] B[b, k, n]) against the CPU oracle, through the C ABI."""
import numpy as np
import pytest

from oracle import gemm_oracle as orc
from paper_2512_09196_amd import tf
from paper_2512_09196_amd import workloads as wl

import gpu_util as gu

pytestmark = pytest.mark.gpu
CANARY = np.float32(-1.2345678e30)


def bound(c, s, K):
    return 2.0 * gu.gamma(K + 1) * s + 2.0 ** -23 * np.abs(c) + 1e-30


def pad_last(bits, ld, rows_stride=None):
    """[batch, R, C] -> [batch, rows_stride or R, ld] with NaN patterns in the padding."""
    nb, R, Cc = bits.shape
    out = np.full((nb, R if rows_stride is None else rows_stride, ld), 0x7FC1, np.uint16)
    out[:, :R, :Cc] = bits
    return out


def check_all(nb, M, N, K, A, B, lda=None, ldb=None, ldy=None, extra_rows=0, exact=False, only=None):
    torch = gu.torch_mod()
    c, s = orc.batched_gemm_tn(A, B)
    lda_, ldb_, ldy_ = lda or M, ldb or N, ldy or N
    rows_a, rows_b, rows_y = K + extra_rows, K + extra_rows, M + extra_rows
    dA = gu.to_dev(pad_last(A, lda_, rows_a))
    dB = gu.to_dev(pad_last(B, ldb_, rows_b))
    Y = torch.full((nb + 2, rows_y, ldy_), float(CANARY), dtype=torch.float32, device="cuda")     # one guard item at each end
    yptr = Y.data_ptr() + rows_y * ldy_ * 4
    ran = []
    with tf.Problem(M, N, K, lda=lda_, ldb=ldb_, ldy=ldy_, op=tf.TF_OP_BATCHED_GEMM_TN, batch=nb,
                    stride_a=rows_a * lda_, stride_b=rows_b * ldb_, stride_y=rows_y * ldy_) as prob:
        for v in prob.variants():
            name = v.name.decode()
            if only is not None and not only(v):
                continue
            print("case", (nb, M, N, K), "variant", name, flush=True)
            Y.fill_(float(CANARY))
            prob.run(v.id, dA, dB, None, yptr)
            torch.cuda.synchronize()
            h = Y.cpu().numpy()
            assert np.all(h[0] == CANARY) and np.all(h[-1] == CANARY), "%s wrote outside C" % name
            body = h[1:-1]
            assert np.all(body[:, M:, :] == CANARY) and np.all(body[:, :, N:] == CANARY), "%s wrote into the padding" % name
            got = body[:, :M, :N].astype(np.float64)
            assert not np.any(body[:, :M, :N] == CANARY), "%s left elements unwritten" % name
            if exact:
                assert np.array_equal(got, c), name
            else:
                err = np.abs(got - c)
                assert np.all(err <= bound(c, s, K)), "%s: worst excess %g" % (name, (err - bound(c, s, K)).max())
            ran.append(name)
    return ran


def test_t1_every_variant():
    w = wl.BGEMM_WORKLOADS["T1"]
    A, B = wl.make_bgemm(w.batch, w.M, w.N, w.K, w.seed)
    ran = check_all(w.batch, w.M, w.N, w.K, A, B)
    assert ran[0] == "bgemm_tn_naive_1elem_per_thread"
    assert any(n.endswith("ldstrans") for n in ran) and any(n.endswith("pretrans") for n in ran)


@pytest.mark.parametrize("shape", [(1, 264, 520, 192), (5, 72, 40, 64), (2, 520, 136, 320), (3, 40, 48, 64), (2, 1032, 264, 128),
                                   (8, 72, 136, 64), (16, 40, 200, 128)])     # batches of 8: items pinned to XCDs
def test_ragged_tiles(shape):
    nb, M, N, K = shape
    A, B = wl.make_bgemm(nb, M, N, K, seed=200 + M)
    ran = check_all(nb, M, N, K, A, B)
    assert any(n.endswith("ldstrans") for n in ran)


@pytest.mark.parametrize("shape", [(2, 40, 24, 96), (1, 17, 19, 23), (3, 16, 16, 8)])
def test_shapes_the_tile_kernels_do_not_take_run_on_the_naive_kernel(shape):
    nb, M, N, K = shape
    A, B = wl.make_bgemm(nb, M, N, K, seed=5 + K)
    ran = check_all(nb, M, N, K, A, B)
    assert ran == ["bgemm_tn_naive_1elem_per_thread"]


@pytest.mark.parametrize("shape", [(3, 256, 384, 192), (16, 128, 128, 128), (9, 256, 128, 256), (1, 128, 256, 512), (40, 128, 128, 192)])
def test_whole_tile_shapes_include_the_persistent_kernels(shape):
    # batches that are and are not multiples of 8, fewer tiles than work-groups and more, 2 to 8 K steps per tile
    nb, M, N, K = shape
    A, B = wl.make_bgemm(nb, M, N, K, seed=300 + nb)
    ran = check_all(nb, M, N, K, A, B)
    assert any(n.endswith("persist") for n in ran)


def test_leading_dimensions_and_item_strides():
    nb, M, N, K = 3, 200, 136, 128
    A, B = wl.make_bgemm(nb, M, N, K, seed=77)
    check_all(nb, M, N, K, A, B, lda=M + 8, ldb=N + 24, ldy=N + 4, extra_rows=3)
    # whole tiles, so that the persistent kernels take part
    nb, M, N, K = 5, 256, 128, 192
    A, B = wl.make_bgemm(nb, M, N, K, seed=78)
    ran = check_all(nb, M, N, K, A, B, lda=M + 8, ldb=N + 24, ldy=N + 4, extra_rows=3)
    assert any(n.endswith("persist") for n in ran)


def test_integer_operands_are_bit_exact():
    nb, M, N, K = 2, 136, 264, 256
    A = wl.small_int_bf16(19, 0, (nb, K, M))
    B = wl.small_int_bf16(19, 1, (nb, K, N))
    check_all(nb, M, N, K, A, B, exact=True)


def test_degenerate_sizes_and_errors():
    with tf.Problem(16, 16, 64, op=tf.TF_OP_BATCHED_GEMM_TN, batch=0) as prob:
        prob.run(0, None, None, None, None)          # nothing to do
    with pytest.raises(tf.TfError):
        tf.Problem(16, 16, 64, lda=8, op=tf.TF_OP_BATCHED_GEMM_TN, batch=1)      # rows of A are M long
    with pytest.raises(tf.TfError):
        tf.Problem(16, 16, 64, op=tf.TF_OP_BATCHED_GEMM_TN, batch=2, stride_y=100)


def test_variant_loop_and_full_size_t2_against_the_whole_oracle():
    torch = gu.torch_mod()
    for name in ("T1", "T2"):
        w = wl.BGEMM_WORKLOADS[name]
        A, B = wl.make_bgemm(w.batch, w.M, w.N, w.K, w.seed)
        c, s = orc.batched_gemm_tn(A, B)
        dA, dB = gu.to_dev(A), gu.to_dev(B)
        Y = torch.empty((w.batch, w.M, w.N), dtype=torch.float32, device="cuda")
        with tf.Problem(w.M, w.N, w.K, op=tf.TF_OP_BATCHED_GEMM_TN, batch=w.batch) as prob:
            if name == "T2":
                for v in prob.variants():
                    if v.kind == tf.TF_KIND_BGEMM_TN_NAIVE:
                        continue
                    print(name, v.name.decode(), flush=True)
                    Y.fill_(float("nan"))
                    prob.run(v.id, dA, dB, None, Y)
                    got = Y.double().cpu().numpy()
                    assert not np.isnan(got).any(), v.name.decode()
                    assert np.all(np.abs(got - c) <= bound(c, s, w.K)), v.name.decode()
            best, rep, log = prob.tune(dA, dB, None, Y)
            print(name, "tune ->", prob.variants()[best].name.decode(), "%.2f us" % rep.t_med_us,
                  "%.0f TFLOP/s %.0f GB/s" % (rep.tflops, rep.gbytes_per_s), "rounds", len(log) - 1, flush=True)
            assert log[0].variant_id == 0 and rep.parity_ok == 1 and rep.status == 0
            assert best != 0 and log[0].t_med_us / rep.t_med_us >= 1.05
            got = Y.double().cpu().numpy()
            assert np.all(np.abs(got - c) <= bound(c, s, w.K))
