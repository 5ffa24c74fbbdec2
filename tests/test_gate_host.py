"""Host-side decisions that guard the GPU path, checked without a GPU:
  * the comparison rule of tf_tune's built-in correctness gate (tf_gate_count_bad is the same rule the
    device kernel applies), on outputs fabricated from the oracle;
  * the decision of the work-group placement probe behind the L2-local split-K reduction;
  * which shapes are offered that reduction at all."""
import math

import numpy as np
import pytest

from oracle import gemm_oracle as orc
from paper_2512_09196_amd import tf
from paper_2512_09196_amd import workloads as wl


def norms(bits, axis):
    x = wl.bf16_bits_to_f32(bits).astype(np.float64)
    return (np.sqrt((x * x).sum(axis=axis)) * 1.0001).astype(np.float32)


def gelu_of(z):
    return np.array([orc.gelu(float(v)) for v in np.ravel(z)]).reshape(np.shape(z))


def case(M, N, K, seed):
    # the recipe of the tall-K workload: uniform operands scaled by 1/sqrt(K), bias ~ N(0, 1)
    A, B, bias = wl.make_custom(M, N, K, seed=seed)
    y, z, s = orc.gemm_bias_gelu(A, B, bias)
    return A, B, bias, y, z, s


def test_gate_accepts_the_rounded_oracle_and_rejects_an_output_without_the_matrix_product():
    M, N, K = 24, 256, 16384
    A, B, bias, y, z, s = case(M, N, K, seed=4)
    na, nb = norms(A, 1), norms(B, 0)
    zref = z.astype(np.float32)
    good = wl.f64_to_bf16_bits(y)
    assert tf.gate_count_bad(good, zref, na, nb, K, tf.TF_EPI_BIAS_GELU_ERF) == 0
    # what a kernel that skipped the K loop would write: GELU(bias) in every row
    b = wl.bf16_bits_to_f32(bias).astype(np.float64)
    skipped = wl.f64_to_bf16_bits(np.broadcast_to(gelu_of(b), (M, N)).copy())
    # ... which the stated tolerance of 1e-2 (1 + |y|) cannot see on this workload
    assert np.all(np.abs(wl.bf16_bits_to_f32(skipped).astype(np.float64) - y) <= 1e-2 * (1 + np.abs(y)))
    bad = tf.gate_count_bad(skipped, zref, na, nb, K, tf.TF_EPI_BIAS_GELU_ERF)
    assert bad > M * N // 100, "the gate must see a missing matrix product (%d rejected)" % bad
    # fp32 output: the pre-activation without the product is the bias alone
    z32 = z.astype(np.float32)
    assert tf.gate_count_bad(z32, zref, na, nb, K, tf.TF_EPI_NONE_F32) == 0
    only_bias = np.broadcast_to(b.astype(np.float32), (M, N)).copy()
    assert tf.gate_count_bad(only_bias, zref, na, nb, K, tf.TF_EPI_NONE_F32) > M * N // 2


def test_gate_rejects_unwritten_and_misplaced_elements():
    M, N, K = 16, 64, 256
    A, B, bias, y, z, s = case(M, N, K, seed=9)
    na, nb = norms(A, 1), norms(B, 0)
    zref = z.astype(np.float32)
    good = wl.f64_to_bf16_bits(y)
    assert tf.gate_count_bad(good, zref, na, nb, K, tf.TF_EPI_BIAS_GELU_ERF) == 0
    one_nan = good.copy()
    one_nan[3, 5] = 0x7FC0
    assert tf.gate_count_bad(one_nan, zref, na, nb, K, tf.TF_EPI_BIAS_GELU_ERF) == 1
    shifted = np.roll(good, 1, axis=1)          # every element one column off
    assert tf.gate_count_bad(shifted, zref, na, nb, K, tf.TF_EPI_BIAS_GELU_ERF) > M * N // 2
    # a strided Y: the padding columns are not looked at
    padded = np.full((M, N + 8), 0x7FC1, np.uint16)
    padded[:, :N] = good
    assert tf.gate_count_bad(padded[:, :N], zref, na, nb, K, tf.TF_EPI_BIAS_GELU_ERF) == 0
    # the tanh form is a different function: its rounded values fail the erf gate somewhere, and pass their own
    ytanh = orc.gelu_tanh(z)
    t = wl.f64_to_bf16_bits(ytanh)
    assert tf.gate_count_bad(t, zref, na, nb, K, tf.TF_EPI_BIAS_GELU_TANH) == 0
    assert tf.gate_count_bad(wl.f64_to_bf16_bits(z), zref, na, nb, K, tf.TF_EPI_BIAS) == 0


def test_gate_bound_is_the_documented_formula():
    # one element, values chosen by hand: K = 255 -> g = 256 * 2^-24 / (1 - 256 * 2^-24)
    K = 255
    g = 256 * 2.0 ** -24 / (1 - 256 * 2.0 ** -24)
    zref = np.array([[1.0]], np.float32)
    na, nb = np.array([2.0], np.float32), np.array([3.0], np.float32)
    tol32 = 3 * g * 6.0 + 2.0 ** -22
    inside = np.array([[1.0 + 0.9 * tol32]], np.float32)
    outside = np.array([[1.0 + 1.2 * tol32]], np.float32)
    assert tf.gate_count_bad(inside, zref, na, nb, K, tf.TF_EPI_NONE_F32) == 0
    assert tf.gate_count_bad(outside, zref, na, nb, K, tf.TF_EPI_NONE_F32) == 1
    ref = 0.8413447460685429         # GELU(1) = Phi(1), from a normal table
    tol16 = 2.0 ** -8 * ref + 1.13 * tol32 + 2e-6 * 2
    def bits(v):
        return wl.f64_to_bf16_bits(np.array([[v]]))
    # bf16 neighbours of GELU(1) are 2^-8 apart: the nearest passes, a value two steps away does not
    assert tf.gate_count_bad(bits(ref), zref, na, nb, K, tf.TF_EPI_BIAS_GELU_ERF) == 0
    assert abs(float(wl.bf16_bits_to_f32(bits(ref + 2.5 * 2.0 ** -8))[0, 0]) - ref) > tol16
    assert tf.gate_count_bad(bits(ref + 2.5 * 2.0 ** -8), zref, na, nb, K, tf.TF_EPI_BIAS_GELU_ERF) == 1


def test_gate_argument_errors():
    z = np.zeros((2, 8), np.float32)
    n = np.ones(8, np.float32)
    with pytest.raises(tf.TfError):
        tf.gate_count_bad(np.zeros((2, 8), np.uint16), z, n, n, -1, tf.TF_EPI_BIAS_GELU_ERF)


def test_placement_probe_decision():
    ok = [i % 8 for i in range(2048)]
    assert tf.xcc_placement_ok(ok)
    # any fixed assignment of the eight residues to XCDs is fine, even a non-bijective one
    perm = [5, 2, 7, 0, 1, 6, 3, 4]
    assert tf.xcc_placement_ok([perm[i % 8] for i in range(512)])
    # a dispatcher that hands out pairs, or skips one XCD once, is not
    assert not tf.xcc_placement_ok([(i // 2) % 8 for i in range(512)])
    broken = list(ok)
    broken[1000] = (broken[1000] + 1) % 8
    assert not tf.xcc_placement_ok(broken)
    # too few work-groups to tell
    assert not tf.xcc_placement_ok(ok[:8])
    assert not tf.xcc_placement_ok([])


def test_l2_local_reduction_is_offered_for_whole_line_rows_only():
    seen_l = 0
    for (M, N, K) in [(16, 8192, 8192), (1024, 1024, 16384), (128, 264, 4096), (16, 2056, 2048), (256, 1032, 4096),
                      (32, 520, 4096), (128, 1024 + 8, 2048), (16, 512, 2048)]:
        with tf.Problem(M, N, K) as p:
            vs = p.variants()
        local = [v for v in vs if v.split_k > 1 and v.fused_reduce == 2]
        for v in local:
            assert v.name.decode().endswith("l")
            tiles = -(-M // v.bm) * -(-N // v.bn)
            assert N % 32 == 0 and tiles % 8 == 0, v.name.decode()
        if N % 32:
            assert not local, "N = %d: rows of the partial sums are not whole 128-byte lines" % N
            assert not any(v.name.decode().endswith("l") for v in vs if v.split_k > 1)
        seen_l += len(local)
        # the counter area is one size for the whole family and holds the status word
        ws = {v.workspace_bytes - (2 if v.stream_k else v.split_k) * M * N * 4 for v in vs if v.workspace_bytes > 0}
        assert len(ws) <= 1 and all(w >= 256 + 8 and w % 256 == 0 for w in ws)
    assert seen_l > 0


def test_round_robin_placement_is_offered_for_one_row_of_tiles_only():
    # tiles dealt round-robin over the XCDs (names with _rr, xcd_swizzle 0) suit problems whose every byte of B is read
    # by one work-group; with several rows of tiles the work-groups of an XCD share panels and keep their contiguous run
    with tf.Problem(16, 8192, 8192) as p:
        vs = p.variants()
        rr = [v for v in vs if v.xcd_swizzle == 0 and v.kind == tf.TF_KIND_MFMA_LDS]
        assert rr and all(b"_rr_" in v.name for v in rr)
        assert all(v.bm >= 16 and -(-16 // v.bm) == 1 for v in rr)
        # each has its twin with the contiguous placement, and the L2-local reduction is still offered (64 or 128 tiles:
        # a multiple of eight, so the slices of a tile stay on one XCD)
        names = {v.name.decode() for v in vs}
        assert all(v.name.decode().replace("_rr_", "_") in names for v in rr)
        assert any(v.fused_reduce == 2 for v in rr)
    with tf.Problem(2048, 2048, 2048) as p:
        assert not [v for v in p.variants() if v.kind == tf.TF_KIND_MFMA_LDS and v.xcd_swizzle == 0]
    with tf.Problem(64, 4096, 4096) as p:
        rr = [v for v in p.variants() if v.kind == tf.TF_KIND_MFMA_LDS and v.xcd_swizzle == 0]
        assert rr and all(v.bm >= 64 for v in rr)          # 64-row tiles: one row of tiles; 32-row tiles: two rows, no _rr
