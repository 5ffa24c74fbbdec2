"""The C boundary without a GPU: the library loads, exports every function include/tf.h
declares, its structs have the layout the binding assumes, enumeration works, and a launch
without a device fails loudly instead of falling back to anything."""
import ctypes
import os
import re
import subprocess
import tempfile

import pytest

from paper_2512_09196_amd import tf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "tf.h")


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(tf_[a-z_0-9]+)\s*\(", src)) - {"tf_parity_fn"})


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(tf.LIB_PATH)
    names = declared_functions()
    assert len(names) >= 20
    for n in names:
        assert hasattr(lib, n), "missing export " + n
    assert set(names) == set(tf.SIGNATURES), "binding and header disagree"


def test_struct_layouts_match_the_header():
    prog = r'''
#include <stdio.h>
#include <stddef.h>
#include "tf.h"
int main(void) {
  printf("%zu %zu %zu %zu %zu\n", sizeof(tf_problem_desc), sizeof(tf_variant_desc), sizeof(tf_report), sizeof(tf_hw), sizeof(tf_theta));
  printf("%zu %zu %zu %zu\n", offsetof(tf_variant_desc, workspace_bytes), offsetof(tf_variant_desc, name),
         offsetof(tf_report, t_min_us), offsetof(tf_report, parity_ok));
  printf("%zu %zu %zu\n", offsetof(tf_report, occupancy_pct), offsetof(tf_hw, clock_mhz), offsetof(tf_theta, cold_bytes));
  return 0;
}'''
    with tempfile.TemporaryDirectory() as d:
        c = os.path.join(d, "t.c")
        open(c, "w").write(prog)
        exe = os.path.join(d, "t")
        subprocess.run(["gcc", "-std=c11", "-I", os.path.join(ROOT, "include"), c, "-o", exe], check=True)
        out = subprocess.run([exe], check=True, stdout=subprocess.PIPE, text=True).stdout.split()
    got = [int(x) for x in out]
    want = [ctypes.sizeof(tf.ProblemDesc), ctypes.sizeof(tf.VariantDesc), ctypes.sizeof(tf.Report),
            ctypes.sizeof(tf.Hw), ctypes.sizeof(tf.Theta),
            tf.VariantDesc.workspace_bytes.offset, tf.VariantDesc.name.offset,
            tf.Report.t_min_us.offset, tf.Report.parity_ok.offset,
            tf.Report.occupancy_pct.offset, tf.Hw.clock_mhz.offset, tf.Theta.cold_bytes.offset]
    assert got == want


def test_enumerate_without_gpu_lists_valid_variants_only():
    with tf.Problem(2048, 2048, 2048) as p:
        vs = p.variants()
    assert vs[0].kind == tf.TF_KIND_NAIVE and vs[0].id == 0
    assert [v.id for v in vs] == list(range(len(vs)))
    names = [v.name.decode() for v in vs]
    assert len(set(names)) == len(names)
    lds = [v for v in vs if v.kind == tf.TF_KIND_MFMA_LDS]
    assert any(v.bm == 256 and v.bn == 256 for v in lds) and any(v.bm == 128 and v.bn == 128 for v in lds)
    for v in lds:
        assert v.lds_bytes <= 160 * 1024 and v.threads == 64 * v.waves_m * v.waves_n * v.waves_k
        tiles = -(-2048 // v.bm) * -(-2048 // v.bn)
        assert v.grid == tiles * v.split_k
        if v.split_k > 1:
            assert v.workspace_bytes >= v.split_k * 2048 * 2048 * 4
        else:
            assert v.workspace_bytes == 0


def test_enumerate_respects_alignment_and_ragged_k():
    # N not a multiple of 8: no 16-byte staging possible -> only the two unstaged kernels
    with tf.Problem(17, 19, 23) as p:
        kinds = [v.kind for v in p.variants()]
    assert kinds == [tf.TF_KIND_NAIVE, tf.TF_KIND_MFMA_DIRECT]
    # K multiple of 8 but not of 64: only register-staged tile kernels (zero fill of the tail)
    with tf.Problem(200, 136, 72) as p:
        lds = [v for v in p.variants() if v.kind == tf.TF_KIND_MFMA_LDS]
    assert lds and all(v.direct_to_lds == 0 for v in lds)
    # skinny decode shape: small-M tiles only, split-K offered
    with tf.Problem(16, 8192, 8192) as p:
        lds = [v for v in p.variants() if v.kind == tf.TF_KIND_MFMA_LDS]
    assert lds and all(v.bm == 32 for v in lds) and any(v.split_k > 1 for v in lds)
    # empty problem
    with tf.Problem(0, 64, 64) as p:
        assert [v.kind for v in p.variants()] == [tf.TF_KIND_NAIVE]


def test_enumerate_the_other_operations_without_gpu():
    hw = tf.hw_nominal()
    # batched vector-matrix product: naive first, then the streaming family at several grid sizes
    with tf.Problem(32, 4096, 4096, op=tf.TF_OP_BATCHED_VECMAT) as p:
        vs = p.variants()
        assert p.desc.ldb == 4096 and p.desc.epi == tf.TF_EPI_NONE_F32
        assert vs[0].kind == tf.TF_KIND_VECMAT_NAIVE
        st = [v for v in vs if v.kind == tf.TF_KIND_VECMAT_STREAM]
        assert len(st) >= 9 and all(v.workspace_bytes == 0 and v.lds_bytes == 0 for v in st)
        for v in st:
            groups = -(-4096 // v.bm) * 32
            full = -(-groups // v.waves_k)
            assert v.grid == (full if v.group_m == 0 else min(full, v.group_m * hw.cus))
        pred = {v.name.decode(): tf.predict_us(p.desc, hw, v) for v in vs}
        assert min(pred.values()) >= 2 * 32 * 4096 * 4096 / 8e12 * 1e6           # never below the HBM roof
        assert pred["vecmat_naive_1elem_per_thread"] > 5 * min(pred.values())
    with tf.Problem(4, 33, 1001, op=tf.TF_OP_BATCHED_VECMAT) as p:          # K not a multiple of 8
        assert [v.kind for v in p.variants()] == [tf.TF_KIND_VECMAT_NAIVE]
    # batched transposed-operand product: transposed staging and the separate-pass alternative
    with tf.Problem(1024, 1024, 256, op=tf.TF_OP_BATCHED_GEMM_TN, batch=32) as p:
        vs = p.variants()
        assert p.desc.lda == 1024 and p.desc.stride_a == 256 * 1024 and p.desc.stride_y == 1024 * 1024
        assert vs[0].kind == tf.TF_KIND_BGEMM_TN_NAIVE
        tiles = [v for v in vs if v.kind == tf.TF_KIND_MFMA_LDS]
        assert any(v.trans_a for v in tiles) and any(not v.trans_a for v in tiles)
        for v in tiles:
            assert v.split_k == 1 and v.direct_to_lds == 1
            assert v.grid == (hw.cus if v.persistent else -(-1024 // v.bm) * -(-1024 // v.bn) * 32)
            assert v.workspace_bytes == (0 if v.trans_a else 32 * 1024 * 256 * 2)
        assert sum(v.persistent for v in tiles) >= 2 and all(v.trans_a and v.stages >= 3 for v in tiles if v.persistent)
        pred = {v.name.decode(): tf.predict_us(p.desc, hw, v) for v in vs}
        best = min(pred, key=pred.get)
        assert not best.endswith("pretrans")                                   # the extra pass is never predicted to pay
    with tf.Problem(40, 24, 96, op=tf.TF_OP_BATCHED_GEMM_TN, batch=2) as p:  # K not a multiple of 64
        assert [v.kind for v in p.variants()] == [tf.TF_KIND_BGEMM_TN_NAIVE]
    # element-wise sine: the four-element baseline first, then one kernel per launch shape, also as a grid-stride launch
    n = 1 << 26
    with tf.Problem(1, n, 0, op=tf.TF_OP_ELEMENTWISE_SIN) as p:
        vs = p.variants()
        assert p.desc.epi == tf.TF_EPI_NONE_F32 and p.desc.N == n
        assert vs[0].name == b"sin_block4_t64" and vs[0].grid == n // 4 and all(v.kind == tf.TF_KIND_SIN for v in vs)
        assert len(vs) >= 15 and len({v.name for v in vs}) == len(vs)
        for v in vs[1:]:
            assert v.bn == v.threads * v.bk * v.stages and v.workspace_bytes == 0 and v.lds_bytes == 0
            full = -(-n // v.bn)
            assert v.grid == (full if v.group_m == 0 else min(full, v.group_m * hw.cus))
        pred = {v.name.decode(): tf.predict_us(p.desc, hw, v) for v in vs}
        assert min(pred.values()) >= 8 * n / 8e12 * 1e6                           # never below the HBM roof
        assert pred["sin_block4_t64"] > 20 * min(pred.values())
        assert min(pred, key=pred.get).split("_")[3] == "v4"
    with tf.Problem(1, 0, 0, op=tf.TF_OP_ELEMENTWISE_SIN) as p:
        assert len(p.variants()) == 1
    with pytest.raises(tf.TfError):
        tf.Problem(1, -1, 0, op=tf.TF_OP_ELEMENTWISE_SIN)
    # every epilogue of the GEMM lists the same family; only the GEMM takes the bf16 ones
    with tf.Problem(2048, 2048, 2048) as p0:
        names = [v.name for v in p0.variants()]
        t_erf = tf.predict_us(p0.desc, hw, p0.variants()[5])
        for epi in (tf.TF_EPI_NONE_F32, tf.TF_EPI_BIAS, tf.TF_EPI_BIAS_GELU_TANH):
            with tf.Problem(2048, 2048, 2048, epi=epi) as p:
                assert [v.name for v in p.variants()] == names
                assert tf.predict_us(p.desc, hw, p.variants()[5]) <= t_erf     # cheaper epilogues are never predicted slower
    # the GEMM never lists kernels of the transposed-operand product
    with tf.Problem(2048, 2048, 2048) as p:
        assert all(v.trans_a == 0 for v in p.variants())
    for bad in (dict(ldb=8, op=tf.TF_OP_BATCHED_VECMAT), dict(lda=8, op=tf.TF_OP_BATCHED_GEMM_TN, batch=1),
                dict(op=tf.TF_OP_BATCHED_GEMM_TN, batch=2, stride_b=10), dict(op=7)):
        with pytest.raises(tf.TfError):
            tf.Problem(16, 16, 64, **bad)


def test_bad_problem_is_rejected():
    with pytest.raises(tf.TfError) as e:
        tf.Problem(-1, 8, 8)
    assert e.value.status == tf.TF_E_INVALID
    with pytest.raises(tf.TfError):
        tf.Problem(8, 8, 8, lda=4)
    with pytest.raises(tf.TfError):
        tf.Problem(8, 8, 8, epi=7)


def test_no_gpu_means_loud_failure_not_fallback():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with tf.Problem(64, 64, 64) as p:
        with pytest.raises(tf.TfError) as e:
            p.run(0, 0x1000, 0x1000, 0x1000, 0x1000, stream=0)
        assert e.value.status == tf.TF_E_LAUNCH
    with pytest.raises(tf.TfError):
        tf.hw_query(0)


def test_nominal_hardware_profile():
    h = tf.hw_nominal()
    assert h.cus == 256 and h.wave_size == 64 and h.lds_bytes_per_cu == 163840
    assert h.bf16_tflops_peak == pytest.approx(2516.6, abs=0.1) and h.hbm_gbs_peak == 8000.0
