"""Parity of the HIP kernels with the CPU oracle, element by element, through the C boundary.

Tolerances:
  official  |gpu - oracle| <= 1e-2 (1 + |oracle|)                      (the stated bar)
  strict    the a-priori bound of a correct fp32-accumulating kernel   (gpu_util.strict_bound)
  exact     bit equality of the fp32 pre-activation on integer-valued operands
"""
import numpy as np
import pytest

from oracle import gemm_oracle as orc
from paper_2512_09196_amd import tf
from paper_2512_09196_amd import workloads as wl

import gpu_util as gu

pytestmark = pytest.mark.gpu


def variants_by_kind(prob):
    return prob.variants()


def check_all_variants(M, N, K, A, B, bias, lda=None, ldb=None, ldy=None, only=None, trans_b=False):
    """Every variant enumerated for the shape against the oracle, with both epilogues.
    trans_b: B is handed over as [N, K] (k contiguous) and checked against the oracle written for that layout."""
    y, z, s = orc.gemm_nt_bias_gelu(A, B, bias) if trans_b else orc.gemm_bias_gelu(A, B, bias)
    dA = gu.to_dev(A if lda is None else gu.strided(A, lda))
    dB = gu.to_dev(B if ldb is None else gu.strided(B, ldb))
    dbias = gu.to_dev(bias)
    ran = []
    for epi, f32 in ((tf.TF_EPI_BIAS_GELU_ERF, False), (tf.TF_EPI_NONE_F32, True)):
        out = gu.OutBuf(M, N, ldy=ldy, f32=f32)
        with tf.Problem(M, N, K, lda=lda, ldb=ldb, ldy=ldy, epi=epi, trans_b=trans_b) as prob:
            for v in prob.variants():
                if only is not None and not only(v):
                    continue
                name = v.name.decode()
                print("case", (M, N, K), "trans_b" if trans_b else "", "epi", epi, "variant", name, flush=True)
                got, intact, _ = gu.run_variant(prob, v.id, dA, dB, dbias, out)
                assert intact, "%s wrote outside Y" % name
                assert not np.isnan(got).any(), "%s left elements unwritten" % name
                if f32:
                    err = np.abs(got - z)
                    assert np.all(err <= gu.preact_bound(z, s, K)), "%s pre-activation off by %g" % (name, err.max())
                else:
                    assert gu.official_ok(got, y), name
                    err = np.abs(got - y)
                    bound = gu.strict_bound(y, z, s, K)
                    assert np.all(err <= bound), "%s: worst excess %g" % (name, (err - bound).max())
                ran.append(name)
                # whatever ran last (a transposing pass into the workspace, a reduction that left its counters
                # behind), the status word of the workspace must still read "no misplaced slice"
                prob.workspace_status()
    return ran


def test_c1_every_variant():
    w = wl.WORKLOADS["C1"]
    A, B, bias = wl.make_inputs(w)
    ran = check_all_variants(w.M, w.N, w.K, A, B, bias)
    assert any(n.startswith("lds_") for n in ran) and "naive_1elem_per_thread" in ran and "mfma32_direct_1wave" in ran


@pytest.mark.parametrize("shape", [(300, 520, 448), (130, 264, 192), (33, 72, 64), (257, 136, 1024)])
def test_ragged_tiles_direct_and_register_staging(shape):
    # several tiles in M and N with a ragged last tile; K a multiple of 64
    M, N, K = shape
    A, B, bias = wl.make_custom(M, N, K, seed=sum(shape))
    ran = check_all_variants(M, N, K, A, B, bias)
    assert any("direct" in n for n in ran) and any("regs" in n for n in ran)


@pytest.mark.parametrize("shape", [(200, 136, 72), (70, 80, 200), (64, 64, 8)])
def test_ragged_k_tail_is_zero_filled(shape):
    M, N, K = shape
    A, B, bias = wl.make_custom(M, N, K, seed=7 + K, a_dist=("normal", 1.0), b_dist=("normal", 0.3))
    ran = check_all_variants(M, N, K, A, B, bias)
    assert any("regs" in n for n in ran) and not any("direct" in n and n.startswith("lds") for n in ran)


@pytest.mark.parametrize("shape", [(17, 19, 23), (1, 1, 1), (5, 3, 100), (40, 33, 7)])
def test_unaligned_shapes_run_on_the_unstaged_kernels(shape):
    M, N, K = shape
    A, B, bias = wl.make_custom(M, N, K, seed=99 + M)
    ran = check_all_variants(M, N, K, A, B, bias)
    assert ran.count("naive_1elem_per_thread") == 2 and ran.count("mfma32_direct_1wave") == 2
    assert not any(n.startswith("lds") for n in ran)


def test_split_k_variants():
    M, N, K = 128, 256, 4096
    A, B, bias = wl.make_custom(M, N, K, seed=5)
    ran = check_all_variants(M, N, K, A, B, bias, only=lambda v: v.kind == tf.TF_KIND_MFMA_LDS)
    assert any("_sk2" in n for n in ran) and any("_sk8" in n or "_sk16" in n for n in ran)


def test_skinny_decode_shape_small():
    M, N, K = 16, 512, 2048
    A, B, bias = wl.make_custom(M, N, K, seed=3, a_dist=("normal", 1.0), b_dist=("normal", 0.02),
                                bias_dist=("normal", 0.01))
    ran = check_all_variants(M, N, K, A, B, bias)
    assert any(n.startswith("lds_32x") for n in ran)


@pytest.mark.parametrize("shape", [(16, 512, 2048), (7, 200, 96), (32, 1000, 4128), (17, 136, 32), (1, 8, 64),
                                   (16, 2056, 1024)])
def test_streaming_kernels_on_skinny_shapes(shape):
    # M <= 32: B streamed once, waves split K; ragged column block, rows past M, K of one block only,
    # uneven runs of K blocks per wave, one- and two-kernel reductions
    M, N, K = shape
    A, B, bias = wl.make_custom(M, N, K, seed=11 + N, a_dist=("normal", 1.0), b_dist=("normal", 0.05),
                                bias_dist=("normal", 0.3))
    ran = check_all_variants(M, N, K, A, B, bias, only=lambda v: v.kind == tf.TF_KIND_MFMA_STREAM)
    assert N <= 64 or any(n.startswith("stream_%dx128x" % (16 if M <= 16 else 32)) for n in ran)
    assert any(n.startswith("stream_%dx64x" % (16 if M <= 16 else 32)) for n in ran)
    if K >= 2048:
        assert any(n.endswith("r") for n in ran)
    # strided operands
    ran = check_all_variants(M, N, K, *wl.make_custom(M, N, K, seed=5 + K), lda=K + 8, ldb=N + 24, ldy=N + 8,
                             only=lambda v: v.kind == tf.TF_KIND_MFMA_STREAM)
    assert ran


def test_leading_dimensions_and_padding_columns():
    M, N, K = 150, 200, 320
    A, B, bias = wl.make_custom(M, N, K, seed=17)
    check_all_variants(M, N, K, A, B, bias, lda=K + 24, ldb=N + 8, ldy=N + 16)


@pytest.mark.parametrize("shape", [(256, 256, 256), (300, 520, 448), (16, 512, 2048), (40, 33, 7), (1024, 1024, 4096)])
def test_bias_only_and_tanh_gelu_epilogues(shape):
    # every variant with the two further bf16 epilogues: Y = bf16(z) and Y = bf16(GELU_tanh(z)), z = A.B + bias
    M, N, K = shape
    A, B, bias = wl.make_custom(M, N, K, seed=91 + M)
    _, z, s = orc.gemm_bias_gelu(A, B, bias)
    dA, dB, dbias = gu.to_dev(A), gu.to_dev(B), gu.to_dev(bias)
    for epi, want in ((tf.TF_EPI_BIAS, z), (tf.TF_EPI_BIAS_GELU_TANH, orc.gelu_tanh(z.ravel()).reshape(z.shape))):
        out = gu.OutBuf(M, N)
        kinds = set()
        with tf.Problem(M, N, K, epi=epi) as prob:
            for v in prob.variants():
                if M >= 1024 and v.kind in (tf.TF_KIND_NAIVE, tf.TF_KIND_MFMA_DIRECT):
                    continue
                name = v.name.decode()
                print("case", shape, "epi", epi, "variant", name, flush=True)
                got, intact, _ = gu.run_variant(prob, v.id, dA, dB, dbias, out)
                assert intact, "%s wrote outside Y" % name
                assert not np.isnan(got).any(), "%s left elements unwritten" % name
                assert gu.official_ok(got, want), name
                err = np.abs(got - want)
                bound = gu.strict_bound(want, z, s, K)      # slope of either function <= 1.13
                assert np.all(err <= bound), "%s: worst excess %g" % (name, (err - bound).max())
                kinds.add(v.kind)
        assert tf.TF_KIND_NAIVE in kinds or M >= 1024


def test_epilogues_differ_where_they_should():
    # guards against an epilogue silently running another one's code
    M, N, K = 128, 128, 64
    A, B, bias = wl.make_custom(M, N, K, seed=5)
    dA, dB, dbias = gu.to_dev(A), gu.to_dev(B), gu.to_dev(bias)
    res = {}
    for epi in (tf.TF_EPI_BIAS_GELU_ERF, tf.TF_EPI_BIAS, tf.TF_EPI_BIAS_GELU_TANH):
        out = gu.OutBuf(M, N)
        with tf.Problem(M, N, K, epi=epi) as prob:
            v = [v for v in prob.variants() if v.kind == tf.TF_KIND_MFMA_LDS][0]
            res[epi], _, _ = gu.run_variant(prob, v.id, dA, dB, dbias, out)
    z = res[tf.TF_EPI_BIAS]
    assert np.any(z < -0.5) and np.all(res[tf.TF_EPI_BIAS_GELU_ERF][z < -0.5] > z[z < -0.5])
    d = np.abs(res[tf.TF_EPI_BIAS_GELU_ERF] - res[tf.TF_EPI_BIAS_GELU_TANH])
    assert d.max() <= 5e-4 + 2.0 ** -7 * np.abs(z).max()          # the two GELUs are close, up to one bf16 step
    assert np.any(d > 0)


@pytest.mark.parametrize("shape", [(2304, 2304, 512), (2200, 2312, 576), (1408, 3200, 1024), (4224, 2176, 512)])
def test_stream_k_variants(shape):
    # between one and three tiles per CU, whole and ragged tiles, both epilogue types; a tile of the shared part
    # has one or two contributors and the result must not depend on who arrives last (run twice, compare bits)
    torch = gu.torch_mod()
    M, N, K = shape
    A, B, bias = wl.make_custom(M, N, K, seed=500 + M)
    ran = check_all_variants(M, N, K, A, B, bias, only=lambda v: v.stream_k == 1)
    assert len(ran) >= 4 and all(n.endswith("streamk") for n in ran)
    dA, dB, dbias = gu.to_dev(A), gu.to_dev(B), gu.to_dev(bias)
    Y1 = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    Y2 = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    with tf.Problem(M, N, K) as prob:
        sk = [v for v in prob.variants() if v.stream_k][0]
        plain = [v for v in prob.variants() if v.kind == tf.TF_KIND_MFMA_LDS and not v.stream_k and v.split_k == 1
                 and v.k_rotate == 0 and (v.bm, v.bn, v.waves_m, v.waves_n, v.waves_k, v.stages) ==
                 (sk.bm, sk.bn, sk.waves_m, sk.waves_n, sk.waves_k, sk.stages)][0]
        for _ in range(3):
            prob.run(sk.id, dA, dB, dbias, Y1)
            prob.run(sk.id, dA, dB, dbias, Y2)
            torch.cuda.synchronize()
            assert torch.equal(Y1.view(torch.int16), Y2.view(torch.int16))
        # against the same kernel without stream-K: tiles computed whole are bit-identical, shared tiles differ
        # by the rounding of one extra fp32 addition at most (then by at most one bf16 step)
        prob.run(plain.id, dA, dB, dbias, Y2)
        torch.cuda.synchronize()
        d = (Y1.float() - Y2.float()).abs()
        assert bool((d <= 2.0 ** -7 * Y2.float().abs() + 1e-6).all().item())
        assert float((d == 0).float().mean().item()) > 0.5


def test_degenerate_sizes():
    torch = gu.torch_mod()
    # K = 0: Y = GELU(bias) on every row
    bias = wl.normal_bf16(1, 2, (24,), 1.0)
    with tf.Problem(6, 24, 0) as prob:
        out = gu.OutBuf(6, 24)
        for v in prob.variants():
            got, intact, _ = gu.run_variant(prob, v.id, 0, 0, gu.to_dev(bias), out)
            want = np.array([orc.gelu(float(b)) for b in wl.bf16_bits_to_f32(bias)])
            assert intact and np.all(np.abs(got - want[None, :]) <= 2.0 ** -8 * np.abs(want) + 1e-6)
    # M = 0 and N = 0: nothing is launched, nothing is written
    for (M, N) in ((0, 16), (16, 0)):
        with tf.Problem(M, N, 64) as prob:
            out = gu.OutBuf(M, max(N, 8))
            prob.run(0, 0, 0, 0, out.ptr)
            torch.cuda.synchronize()
            assert out.host()[1]
    # GELU(0) = 0: all-zero operands give an all-zero (+0) output
    Z = np.zeros((64, 64), np.uint16)
    with tf.Problem(64, 64, 64) as prob:
        out = gu.OutBuf(64, 64)
        for v in prob.variants():
            _, intact, raw = gu.run_variant(prob, v.id, gu.to_dev(Z), gu.to_dev(Z), gu.to_dev(np.zeros(64, np.uint16)), out)
            assert intact and np.all(raw == 0)


def test_integer_operands_are_bit_exact_in_every_variant():
    # |a|,|b| <= 2, K = 1024: every partial sum is an integer below 2^24, so fp32 accumulation is
    # exact in any order -- tile edges, K slices, MFMA lane maps and swizzles all have to be right
    for (M, N, K) in ((192, 320, 1024), (130, 264, 4096), (32, 128, 2048)):
        A = wl.small_int_bf16(41, 0, (M, K))
        B = wl.small_int_bf16(41, 1, (K, N))
        bias = wl.small_int_bf16(41, 2, (N,), -3, 3)
        _, z, _ = orc.gemm_bias_gelu(A, B, bias)
        zf = z.astype(np.float32)
        assert np.array_equal(zf.astype(np.float64), z)
        dA, dB, dbias = gu.to_dev(A), gu.to_dev(B), gu.to_dev(bias)
        out = gu.OutBuf(M, N, f32=True)
        with tf.Problem(M, N, K, epi=tf.TF_EPI_NONE_F32) as prob:
            vs = prob.variants()
            assert any(v.split_k > 1 for v in vs)
            for v in vs:
                print("exact", (M, N, K), v.name.decode(), flush=True)
                _, intact, raw = gu.run_variant(prob, v.id, dA, dB, dbias, out)
                assert intact
                assert np.array_equal(raw, zf), v.name.decode()


def test_identity_and_structured_operands():
    K = N = 128
    _, B, bias = wl.make_custom(K, N, K, seed=23, b_dist=("normal", 1.0))
    A = wl.f64_to_bf16_bits(np.eye(K))
    y, z, s = orc.gemm_bias_gelu(A, B, bias)
    dA, dB, dbias = gu.to_dev(A), gu.to_dev(B), gu.to_dev(bias)
    out = gu.OutBuf(K, N, f32=True)
    with tf.Problem(K, N, K, epi=tf.TF_EPI_NONE_F32) as prob:
        for v in prob.variants():
            _, intact, raw = gu.run_variant(prob, v.id, dA, dB, dbias, out)
            # A = I: z = b + bias, one fp32 addition of two bf16 values
            want = (wl.bf16_bits_to_f32(B) + wl.bf16_bits_to_f32(bias)[None, :]).astype(np.float32)
            assert intact and np.array_equal(raw, want), v.name.decode()


def test_split_k_is_deterministic_and_counters_self_clean():
    M, N, K = 128, 128, 8192
    A, B, bias = wl.make_custom(M, N, K, seed=31)
    dA, dB, dbias = gu.to_dev(A), gu.to_dev(B), gu.to_dev(bias)
    out = gu.OutBuf(M, N, f32=True)
    with tf.Problem(M, N, K, epi=tf.TF_EPI_NONE_F32) as prob:
        sk = [v for v in prob.variants() if v.split_k >= 4]
        assert sk
        for v in sk[:4]:
            first = None
            for rep in range(4):
                _, intact, raw = gu.run_variant(prob, v.id, dA, dB, dbias, out)
                assert intact
                if first is None:
                    first = raw
                assert np.array_equal(raw, first), "run %d of %s differs" % (rep, v.name.decode())


def test_l2_local_reduction_equals_the_two_kernel_reduction_bit_for_bit():
    # fused_reduce 2 keeps the partial tiles in the L2 of the XCD all slices of a tile run on; it sums
    # the slices in the same order as the reduce kernel, so the fp32 pre-activations must be identical,
    # launch after launch, also right after other variants have used the same workspace
    for (M, N, K) in ((512, 512, 4096), (16, 1024, 4096), (1024, 256, 2048)):
        A, B, bias = wl.make_custom(M, N, K, seed=61 + M, a_dist=("normal", 1.0), b_dist=("normal", 0.05))
        dA, dB, dbias = gu.to_dev(A), gu.to_dev(B), gu.to_dev(bias)
        out = gu.OutBuf(M, N, f32=True)
        with tf.Problem(M, N, K, epi=tf.TF_EPI_NONE_F32) as prob:
            by_name = {v.name.decode(): v for v in prob.variants()}
            local = [n for n, v in by_name.items() if v.split_k > 1 and v.fused_reduce == 2]
            assert local, "no variant with the L2-local reduction for %s" % ((M, N, K),)
            for rep in range(2):
                for n in local:
                    twin = by_name[n[:-1] + "r"]
                    print("case", (M, N, K), n, "rep", rep, flush=True)
                    _, ok1, raw_l = gu.run_variant(prob, by_name[n].id, dA, dB, dbias, out)
                    _, ok2, raw_r = gu.run_variant(prob, twin.id, dA, dB, dbias, out)
                    assert ok1 and ok2 and not np.isnan(raw_l).any(), n
                    assert np.array_equal(raw_l, raw_r), n


def test_split_k_variants_with_different_tile_counts_share_one_workspace():
    # tile shapes with 4, 8, 16 and 64 output tiles take turns on the problem's workspace:
    # the partial sums of one must never land on the arrival counters of another
    M, N, K = 512, 512, 2048
    A, B, bias = wl.make_custom(M, N, K, seed=43)
    y, z, s = orc.gemm_bias_gelu(A, B, bias)
    dA, dB, dbias = gu.to_dev(A), gu.to_dev(B), gu.to_dev(bias)
    out = gu.OutBuf(M, N)
    with tf.Problem(M, N, K) as prob:
        sk = [v for v in prob.variants() if v.split_k > 1]
        assert len({(v.bm, v.bn) for v in sk}) >= 3
        for order in (sk, sk[::-1], sk[::3] + sk[1::3] + sk[2::3]):
            for v in order:
                got, intact, _ = gu.run_variant(prob, v.id, dA, dB, dbias, out)
                assert intact and not np.isnan(got).any(), v.name.decode()
                assert np.all(np.abs(got - y) <= gu.strict_bound(y, z, s, K)), v.name.decode()


def test_caller_workspace_and_errors():
    torch = gu.torch_mod()
    M, N, K = 128, 128, 2048
    A, B, bias = wl.make_custom(M, N, K, seed=37)
    y, z, s = orc.gemm_bias_gelu(A, B, bias)
    dA, dB, dbias = gu.to_dev(A), gu.to_dev(B), gu.to_dev(bias)
    out = gu.OutBuf(M, N)
    with tf.Problem(M, N, K) as prob:
        v = [v for v in prob.variants() if v.split_k > 1][0]
        biggest = max(x.workspace_bytes for x in prob.variants())
        ws = torch.full((biggest // 4 + 64,), -1, dtype=torch.int32, device="cuda")   # dirty on purpose
        got, intact, _ = gu.run_variant(prob, v.id, dA, dB, dbias, out, workspace=ws, workspace_bytes=ws.numel() * 4)
        assert intact and np.all(np.abs(got - y) <= gu.strict_bound(y, z, s, K))
        got2, _, _ = gu.run_variant(prob, v.id, dA, dB, dbias, out, workspace=ws, workspace_bytes=ws.numel() * 4)
        assert np.array_equal(got, got2)
        # what a caller's workspace holds between two calls is the caller's: every reduction mode must cope with
        # counters that were overwritten since the last launch (the library zeroes them ahead of each launch)
        modes = set()
        for v2 in [x for x in prob.variants() if x.split_k > 1]:
            for fill in (-1, 0x01010101):
                ws.fill_(fill)
                got3, intact, _ = gu.run_variant(prob, v2.id, dA, dB, dbias, out, workspace=ws, workspace_bytes=ws.numel() * 4)
                assert intact and not np.isnan(got3).any(), v2.name.decode()
                assert np.all(np.abs(got3 - y) <= gu.strict_bound(y, z, s, K)), v2.name.decode()
            modes.add(v2.fused_reduce)
            prob.workspace_status(ws)          # synchronises; raises if an L2-local reduction reported misplaced slices
        assert modes == {0, 1, 2}
        prob.workspace_status()                # the library's own buffer (never used here): nothing to report
        with pytest.raises(tf.TfError) as e:
            prob.run(v.id, dA, dB, dbias, out.ptr, workspace=ws, workspace_bytes=1024)
        assert e.value.status == tf.TF_E_UNSUPPORTED
        with pytest.raises(tf.TfError) as e:
            prob.run(len(prob.variants()), dA, dB, dbias, out.ptr)
        assert e.value.status == tf.TF_E_INVALID
        lds = [v for v in prob.variants() if v.kind == tf.TF_KIND_MFMA_LDS][0]
        with pytest.raises(tf.TfError) as e:
            prob.run(lds.id, dA.data_ptr() + 2, dB, dbias, out.ptr)      # misaligned A
        assert e.value.status == tf.TF_E_UNSUPPORTED
        torch.cuda.synchronize()


def make_nk(M, N, K, seed, **kw):
    """Operands of the custom recipe with B laid out as [N, K]."""
    A, B, bias = wl.make_custom(M, N, K, seed=seed, **kw)
    return A, np.ascontiguousarray(B.T), bias


@pytest.mark.parametrize("shape", [(256, 256, 256), (300, 520, 448), (130, 264, 192), (33, 72, 64), (16, 512, 2048),
                                   (257, 136, 1024), (512, 512, 1024)])
def test_b_given_as_n_by_k(shape):
    # every variant offered for the [N][K] layout: kernels that stage B as it lies (names with _bnk), ordinary kernels
    # behind a transposing pass (_pretransB), and the two unstaged kernels; whole and ragged tiles, split-K
    M, N, K = shape
    A, Bt, bias = make_nk(M, N, K, seed=300 + M)
    ran = check_all_variants(M, N, K, A, Bt, bias, trans_b=True)
    assert any("_bnk_" in n for n in ran) and any("_pretransB_" in n for n in ran)
    assert "naive_1elem_per_thread" in ran and "mfma32_direct_1wave" in ran
    assert not any(n.startswith("stream_") for n in ran)
    if K >= 1024:
        assert any("_bnk_sk2" in n or "_bnk_sk4" in n for n in ran)


def test_b_given_as_n_by_k_strided_ragged_k_and_exact():
    # leading dimensions with padding (NaN patterns behind every row end)
    M, N, K = 150, 200, 320
    A, Bt, bias = make_nk(M, N, K, seed=317)
    ran = check_all_variants(M, N, K, A, Bt, bias, lda=K + 24, ldb=K + 8, ldy=N + 16, trans_b=True)
    assert any("_bnk_" in n for n in ran)
    # K not a multiple of the K tile: the kernels that stage through registers fill the tail with zeros; the direct
    # path is not offered
    M, N, K = 70, 80, 200
    A, Bt, bias = make_nk(M, N, K, seed=318)
    ran = check_all_variants(M, N, K, A, Bt, bias, trans_b=True)
    assert "naive_1elem_per_thread" in ran and any("_regs_bnk_" in n for n in ran) and not any(n.startswith("lds_") and "_direct" in n for n in ran)
    # integer operands: every partial sum is exact in fp32, so the pre-activation must equal the oracle bit for bit
    for (M, N, K) in ((192, 320, 1024), (130, 264, 4096), (32, 128, 2048)):
        A = wl.small_int_bf16(43, 0, (M, K))
        Bt = wl.small_int_bf16(43, 1, (N, K))
        bias = wl.small_int_bf16(43, 2, (N,), -3, 3)
        _, z, _ = orc.gemm_nt_bias_gelu(A, Bt, bias)
        zf = z.astype(np.float32)
        dA, dB, dbias = gu.to_dev(A), gu.to_dev(Bt), gu.to_dev(bias)
        out = gu.OutBuf(M, N, f32=True)
        with tf.Problem(M, N, K, epi=tf.TF_EPI_NONE_F32, trans_b=1) as prob:
            vs = prob.variants()
            assert any(v.split_k > 1 and v.trans_b for v in vs)
            for v in vs:
                print("exact nk", (M, N, K), v.name.decode(), flush=True)
                _, intact, raw = gu.run_variant(prob, v.id, dA, dB, dbias, out)
                assert intact
                assert np.array_equal(raw, zf), v.name.decode()


def test_loop_on_b_given_as_n_by_k():
    torch = gu.torch_mod()
    M, N, K = 1024, 1024, 1024
    A, Bt, bias = make_nk(M, N, K, seed=321)
    y, z, s = orc.gemm_nt_bias_gelu(A, Bt, bias)
    dA, dB, dbias = gu.to_dev(A), gu.to_dev(Bt), gu.to_dev(bias)
    Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    with tf.Problem(M, N, K, trans_b=1) as prob:
        best, rep, log = prob.tune(dA, dB, dbias, Y)
        names = [prob.variants()[r.variant_id].name.decode() for r in log]
        print("loop on [N][K]:", names, "->", names[[r.variant_id for r in log].index(best)], "%.2f us" % rep.t_med_us, flush=True)
        assert best != 0 and rep.parity_ok == 1
        assert all(r.parity_ok == 1 for r in log if r.status == 0)
        got = Y.float().double().cpu().numpy()
        assert np.all(np.abs(got - y) <= gu.strict_bound(y, z, s, K))


@pytest.mark.parametrize("shape", [(2048, 13824, 128), (2048, 13784, 192), (2024, 13824, 64), (4096, 6912, 64)])
def test_launch_with_a_lighter_last_round(shape):
    # whole rounds of 256 x 256 tiles over the leading columns, then one round of tiles that multiply 192 of their 256
    # columns and share out the rest of every row panel: five or six blocks of 32 columns each, the last one possibly
    # cut by N, the last row panel possibly ragged; integer operands, so every element must be exact, and every
    # element must be written exactly by the tile it belongs to
    M, N, K = shape
    A = wl.small_int_bf16(77, 0, (M, K))
    B = wl.small_int_bf16(77, 1, (K, N))
    bias = wl.small_int_bf16(77, 2, (N,), -3, 3)
    _, z, _ = orc.gemm_bias_gelu(A, B, bias)
    zf = z.astype(np.float32)
    assert np.array_equal(zf.astype(np.float64), z)
    dA, dB, dbias = gu.to_dev(A), gu.to_dev(B), gu.to_dev(bias)
    out = gu.OutBuf(M, N, f32=True)
    with tf.Problem(M, N, K, epi=tf.TF_EPI_NONE_F32) as prob:
        tail = [v for v in prob.variants() if v.bn_tail]
        assert len(tail) >= 2 and all(v.grid % 256 == 0 and v.bn_tail == 192 for v in tail)
        for v in tail:
            print("tail", shape, v.name.decode(), flush=True)
            _, intact, raw = gu.run_variant(prob, v.id, dA, dB, dbias, out)
            assert intact
            assert np.array_equal(raw, zf), v.name.decode()
    # the bf16 epilogue through the same variants, against the oracle's bound, on the workload recipe
    A, B, bias = wl.make_custom(M, N, K, seed=78)
    ran = check_all_variants(M, N, K, A, B, bias, only=lambda v: v.bn_tail > 0)
    assert len(ran) >= 4


@pytest.mark.parametrize("shape", [(2048, 13824, 128), (2024, 13784, 64)])
def test_launch_with_a_lighter_last_round_b_given_as_n_by_k(shape):
    # the same launch with B handed over as [N][K] and staged as it lies: integer operands bit for bit, then the bf16
    # epilogue against the oracle written for that layout
    M, N, K = shape
    A = wl.small_int_bf16(77, 0, (M, K))
    Bt = np.ascontiguousarray(wl.small_int_bf16(77, 1, (K, N)).T)
    bias = wl.small_int_bf16(77, 2, (N,), -3, 3)
    _, z, _ = orc.gemm_nt_bias_gelu(A, Bt, bias)
    zf = z.astype(np.float32)
    assert np.array_equal(zf.astype(np.float64), z)
    dA, dB, dbias = gu.to_dev(A), gu.to_dev(Bt), gu.to_dev(bias)
    out = gu.OutBuf(M, N, f32=True)
    with tf.Problem(M, N, K, epi=tf.TF_EPI_NONE_F32, trans_b=1) as prob:
        tail = [v for v in prob.variants() if v.bn_tail]
        assert len(tail) >= 2 and all(v.grid % 256 == 0 and v.bn_tail == 192 and v.trans_b == 1 and b"_bnk_" in v.name for v in tail)
        for v in tail:
            print("tail", shape, v.name.decode(), flush=True)
            _, intact, raw = gu.run_variant(prob, v.id, dA, dB, dbias, out)
            assert intact
            assert np.array_equal(raw, zf), v.name.decode()
    A, B, bias = wl.make_custom(M, N, K, seed=78)
    ran = check_all_variants(M, N, K, A, np.ascontiguousarray(B.T), bias, only=lambda v: v.bn_tail > 0, trans_b=True)
    assert len(ran) >= 4


def test_seeded_random_shapes_every_variant_both_layouts():
    # shapes drawn from a fixed seed: M anything, N and K multiples of 8 (what the tile kernels accept), sizes that
    # span one to several tiles of every tile shape with ragged last tiles in all three dimensions
    rng = np.random.default_rng(20251209)
    total = 0
    for case in range(10):
        M = int(rng.integers(1, 600))
        N = 8 * int(rng.integers(1, 80))
        K = 8 * int(rng.integers(1, 160))
        trans_b = bool(case % 2)
        A, B, bias = wl.make_custom(M, N, K, seed=500 + case)
        if trans_b:
            B = np.ascontiguousarray(B.T)
        ran = check_all_variants(M, N, K, A, B, bias, trans_b=trans_b)
        assert len(ran) >= 4
        total += len(ran)
    print("variants checked:", total, flush=True)
    assert total >= 200
