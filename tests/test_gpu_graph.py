"""tf_variant_run under HIP graph capture: after one eager call (which allocates the workspace and sets the
kernel attributes) a launch records nothing but kernels, so it can be captured and replayed."""
import numpy as np
import pytest

from paper_2512_09196_amd import tf
from paper_2512_09196_amd import workloads as wl

import gpu_util as gu

pytestmark = pytest.mark.gpu


def pick(prob, pred):
    vs = [v for v in prob.variants() if pred(v)]
    assert vs
    return vs[0]


@pytest.mark.parametrize("which", ["plain", "split_two_kernel", "split_in_kernel", "split_l2_local", "stream", "b_as_nk_staged",
                                   "b_as_nk_transposing_pass"])
def test_captured_launches_replay_to_the_eager_result(which):
    torch = gu.torch_mod()
    M, N, K = (16, 512, 4096) if which == "stream" else (256, 256, 2048)
    A, B, bias = wl.make_custom(M, N, K, seed=7)
    nk = which.startswith("b_as_nk")
    if nk:
        B = np.ascontiguousarray(B.T)
    dA, dB, dbias = gu.to_dev(A), gu.to_dev(B), gu.to_dev(bias)
    Y_eager = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
    Y_graph = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
    with tf.Problem(M, N, K, trans_b=1 if nk else 0) as prob:
        v = pick(prob, {
            "plain": lambda v: v.kind == tf.TF_KIND_MFMA_LDS and v.split_k == 1,
            "split_two_kernel": lambda v: v.kind == tf.TF_KIND_MFMA_LDS and v.split_k > 1 and v.fused_reduce == 0,
            "split_in_kernel": lambda v: v.kind == tf.TF_KIND_MFMA_LDS and v.split_k > 1 and v.fused_reduce == 1,
            "split_l2_local": lambda v: v.kind == tf.TF_KIND_MFMA_LDS and v.split_k > 1 and v.fused_reduce == 2,
            "stream": lambda v: v.kind == tf.TF_KIND_MFMA_STREAM and v.split_k > 1,
            "b_as_nk_staged": lambda v: v.kind == tf.TF_KIND_MFMA_LDS and v.trans_b == 1,
            "b_as_nk_transposing_pass": lambda v: b"_pretransB_" in v.name,
        }[which])
        print(which, v.name.decode(), flush=True)
        prob.run(v.id, dA, dB, dbias, Y_eager)                  # eager: first use allocates and sets attributes
        torch.cuda.synchronize()
        want = Y_eager.view(torch.int16).cpu().numpy().copy()
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(s):
            prob.run(v.id, dA, dB, dbias, Y_graph, stream=s)     # same workspace, now known to the problem
            torch.cuda.synchronize()
            Y_graph.zero_()
            with torch.cuda.graph(g, stream=s):
                for _ in range(3):
                    prob.run(v.id, dA, dB, dbias, Y_graph, stream=s)
        for rep in range(4):
            Y_graph.zero_()
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            got = Y_graph.view(torch.int16).cpu().numpy()
            assert np.array_equal(got, want), "replay %d differs from the eager result" % rep
            # eager work of the same problem between the replays (it shares the workspace and its counters)
            prob.run(v.id, dA, dB, dbias, Y_eager)
            torch.cuda.synchronize()
            assert np.array_equal(Y_eager.view(torch.int16).cpu().numpy(), want)
