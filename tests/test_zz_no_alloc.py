"""tf_variant_run_static, the entry point for callers that cannot allocate: the same kernels on the workspace
that is part of the library's device image. Its output must equal tf_variant_run's bit for bit (the split-K
reductions sum in a fixed order), on two calls in a row, the second with a smaller input that leaves most of
the buffer holding the first call's partial sums."""
import numpy as np
import pytest

from oracle import gemm_oracle as orc
from paper_2512_09196_amd import tf
from paper_2512_09196_amd import workloads as wl

import gpu_util as gu

pytestmark = pytest.mark.gpu


def compare_entry_points(M, N, K, seed, check_oracle):
    torch = gu.torch_mod()
    A, B, bias = wl.make_custom(M, N, K, seed=seed)
    dA, dB, dbias = gu.to_dev(A), gu.to_dev(B), gu.to_dev(bias)
    Y1 = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    Y2 = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    cap = tf.lib().tf_static_scratch_bytes()
    modes = set()
    with tf.Problem(M, N, K) as prob:
        vs = [v for v in prob.variants() if v.kind in (tf.TF_KIND_MFMA_LDS, tf.TF_KIND_MFMA_STREAM)]
        split = [v for v in vs if v.workspace_bytes > 0]
        assert split
        # every reduction mode at several slice counts, and a few kernels that need no workspace at all
        todo = split[:: max(1, len(split) // 24)] + [v for v in vs if v.workspace_bytes == 0][:3]
        for v in todo:
            name = v.name.decode()
            print("no-alloc", (M, N, K), name, flush=True)
            if v.workspace_bytes > cap:
                with pytest.raises(tf.TfError) as e:
                    prob.run_static(v.id, dA, dB, dbias, Y2)
                assert e.value.status == tf.TF_E_UNSUPPORTED
                continue
            Y1.fill_(float("nan"))
            Y2.fill_(float("nan"))
            prob.run(v.id, dA, dB, dbias, Y1)
            prob.run_static(v.id, dA, dB, dbias, Y2)
            torch.cuda.synchronize()
            a, b = Y1.view(torch.int16).cpu().numpy(), Y2.view(torch.int16).cpu().numpy()
            assert not np.isnan(Y2.float().cpu().numpy()).any(), name + " left elements unwritten"
            assert np.array_equal(a, b), name
            # again, right away: the counters left by the first call are cleared by the entry point itself
            Y2.fill_(float("nan"))
            prob.run_static(v.id, dA, dB, dbias, Y2)
            torch.cuda.synchronize()
            assert np.array_equal(a, Y2.view(torch.int16).cpu().numpy()), name + " (second call)"
            modes.add((v.split_k > 1, v.fused_reduce))
        if check_oracle:
            y, z, s = orc.gemm_bias_gelu(A, B, bias)
            got = Y2.float().double().cpu().numpy()
            assert np.all(np.abs(got - y) <= gu.strict_bound(y, z, s, K))
    return modes


def test_static_workspace_entry_point_matches_tf_variant_run():
    assert tf.lib().tf_static_scratch_bytes() >= 32 << 20
    big = compare_entry_points(512, 1024, 4096, seed=71, check_oracle=False)
    small = compare_entry_points(96, 256, 2048, seed=72, check_oracle=True)
    # two-kernel reduction in both; in-kernel reduction through the L2 (big: every tile shape gives a multiple of
    # eight tiles) and through memory (small)
    assert (True, 0) in big and (True, 2) in big, big
    assert (True, 0) in small and (True, 1) in small, small


def test_static_workspace_entry_point_rejects_what_does_not_fit():
    torch = gu.torch_mod()
    M = N = 2048
    K = 4096
    dA = torch.zeros((M, K), dtype=torch.int16, device="cuda")
    dB = torch.zeros((K, N), dtype=torch.int16, device="cuda")
    dbias = torch.zeros((N,), dtype=torch.int16, device="cuda")
    Y = torch.full((M, N), 7.0, dtype=torch.bfloat16, device="cuda")
    with tf.Problem(M, N, K) as prob:
        too_big = [v for v in prob.variants() if v.workspace_bytes > tf.lib().tf_static_scratch_bytes()]
        assert too_big
        with pytest.raises(tf.TfError) as e:
            prob.run_static(too_big[0].id, dA, dB, dbias, Y)
        assert e.value.status == tf.TF_E_UNSUPPORTED
        torch.cuda.synchronize()
        assert bool((Y == 7.0).all().item()), "nothing may be launched on an error"
        fits = [v for v in prob.variants() if v.split_k == 2 and v.workspace_bytes <= tf.lib().tf_static_scratch_bytes()]
        if fits:
            prob.run_static(fits[0].id, dA, dB, dbias, Y)
            torch.cuda.synchronize()
            assert bool((Y == 0.0).all().item())       # GELU(0) = 0
