"""Seeded random shapes through a spread of variants and all four epilogues, element by element against the
oracle: a net for tile-edge and addressing mistakes that the hand-picked shapes might miss."""
import numpy as np
import pytest

from oracle import gemm_oracle as orc
from paper_2512_09196_amd import tf
from paper_2512_09196_amd import workloads as wl

import gpu_util as gu

pytestmark = pytest.mark.gpu

EPIS = (tf.TF_EPI_BIAS_GELU_ERF, tf.TF_EPI_NONE_F32, tf.TF_EPI_BIAS, tf.TF_EPI_BIAS_GELU_TANH)


def shapes():
    rng = np.random.default_rng(20251209)
    out = []
    for i in range(24):
        M = int(rng.integers(1, 700))
        N = 8 * int(rng.integers(1, 90))
        K = 8 * int(rng.integers(1, 160))
        out.append((M, N, K, int(rng.integers(0, 3)) * 8, int(rng.integers(0, 3)) * 8, int(rng.integers(0, 3)) * 8))
    return out


@pytest.mark.parametrize("case", shapes())
def test_random_shape(case):
    M, N, K, pa, pb, py = case
    A, B, bias = wl.make_custom(M, N, K, seed=1000 + M + N + K)
    y, z, s = orc.gemm_bias_gelu(A, B, bias)
    want = {tf.TF_EPI_BIAS_GELU_ERF: y, tf.TF_EPI_NONE_F32: z, tf.TF_EPI_BIAS: z,
            tf.TF_EPI_BIAS_GELU_TANH: orc.gelu_tanh(z.ravel()).reshape(z.shape)}
    dA, dB, dbias = gu.to_dev(gu.strided(A, K + pa)), gu.to_dev(gu.strided(B, N + pb)), gu.to_dev(bias)
    for j, epi in enumerate(EPIS):
        f32 = epi == tf.TF_EPI_NONE_F32
        out = gu.OutBuf(M, N, ldy=N + py, f32=f32)
        with tf.Problem(M, N, K, lda=K + pa, ldb=N + pb, ldy=N + py, epi=epi) as prob:
            vs = prob.variants()
            tiles = [v for v in vs if v.kind in (tf.TF_KIND_MFMA_LDS, tf.TF_KIND_MFMA_STREAM)]
            assert tiles, "N and K are multiples of 8: the tile kernels must be offered"
            pick = tiles[j::max(1, len(tiles) // 6)][:7]      # a different spread of the family for each epilogue
            for v in pick:
                name = v.name.decode()
                print("case", case, "epi", epi, "variant", name, flush=True)
                got, intact, _ = gu.run_variant(prob, v.id, dA, dB, dbias, out)
                assert intact, "%s wrote outside Y" % name
                assert not np.isnan(got).any(), "%s left elements unwritten" % name
                err = np.abs(got - want[epi])
                bound = gu.preact_bound(z, s, K) if f32 else gu.strict_bound(want[epi], z, s, K)
                assert np.all(err <= bound), "%s: worst excess %g" % (name, (err - bound).max())


def skinny_shapes():
    """One row of tiles (M <= 32) and a whole number of 64-column tiles: the shapes that are offered the round-robin
    placement over the XCDs, the K tiles dealt to the slices in turn and the L2-local reduction."""
    rng = np.random.default_rng(20251210)
    out = []
    for i in range(8):
        # every other N a multiple of 1024: tile counts that are multiples of eight (what the L2-local reduction needs)
        N = 1024 * int(rng.integers(1, 9)) if i % 4 < 2 else 64 * int(rng.integers(1, 129))
        out.append((int(rng.integers(1, 33)), N, 64 * int(rng.integers(1, 65)), i % 2))
    return out


@pytest.mark.parametrize("case", skinny_shapes())
def test_random_skinny_shape_every_tile_variant(case):
    M, N, K, b_as_nk = case
    A, B, bias = wl.make_custom(M, N, K, seed=2000 + M + N + K)
    y, z, s = orc.gemm_bias_gelu(A, B, bias)
    dA, dbias = gu.to_dev(A), gu.to_dev(bias)
    dB = gu.to_dev(np.ascontiguousarray(B.T)) if b_as_nk else gu.to_dev(B)
    out = gu.OutBuf(M, N)
    bound = gu.strict_bound(y, z, s, K)
    with tf.Problem(M, N, K, trans_b=b_as_nk) as prob:
        tiles = [v for v in prob.variants() if v.kind in (tf.TF_KIND_MFMA_LDS, tf.TF_KIND_MFMA_STREAM)]
        assert tiles
        for v in tiles:
            name = v.name.decode()
            print("case", case, "variant", name, flush=True)
            got, intact, _ = gu.run_variant(prob, v.id, dA, dB, dbias, out)
            assert intact, "%s wrote outside Y" % name
            assert not np.isnan(got).any(), "%s left elements unwritten" % name
            err = np.abs(got - y)
            assert np.all(err <= bound), "%s: worst excess %g" % (name, (err - bound).max())
            prob.workspace_status()
