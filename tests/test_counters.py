"""tf_report_set_counters on rocprofv3 counter files cut from real profiler output (tests/golden/rocprofv3_pmc_*.csv:
the first dispatches of the tile kernels on the 4096 x 11008 x 4096 and 1024 x 1024 x 16384 workloads, plus one
dispatch of another kernel each). The expected figures are worked out by hand from the rows of the files."""
import os

import pytest

from paper_2512_09196_amd import tf

G = os.path.join(os.path.dirname(__file__), "golden")
SQ_C3 = os.path.join(G, "rocprofv3_pmc_sq_C3.csv")
TCC_C3 = os.path.join(G, "rocprofv3_pmc_tcc_C3.csv")
FETCH_C5 = os.path.join(G, "rocprofv3_pmc_fetch_C5.csv")
WRITE_C5 = os.path.join(G, "rocprofv3_pmc_write_C5.csv")


def blank_report(**kw):
    r = tf.Report()
    r.status, r.t_med_us, r.t_min_us, r.grid_fill, r.arithmetic_intensity, r.occupancy_pct = 0, 300.0, 299.0, 0.9, 1727.0, 25.0
    for k, v in kw.items():
        setattr(r, k, v)
    return r


def test_compute_counters_of_the_large_tile_kernel():
    hw = tf.hw_nominal()            # 256 CUs x 4 SIMDs, 8 XCDs, 8 wave slots per SIMD
    r = blank_report(pct_mfma_peak=80.0)
    assert tf.refine_hint(None, r, hw) == tf.TF_BN_MFMA          # what the achieved rate alone would say
    tf.report_set_counters(r, hw, SQ_C3, "LdsCfg<256, 256, 2, 4, 2, true")
    assert r.have_counters == 1
    # two dispatches. GRBM_GUI_ACTIVE: (4840872 + 4581640) / 2 = 4711256 summed over 8 XCDs -> 588907 cycles each
    wall = 4711256.0 / 8
    # SQ_VALU_MFMA_BUSY_CYCLES 360710144 (both dispatches) over 1024 SIMDs
    assert r.mfma_busy_pct == pytest.approx(100 * 360710144.0 / (wall * 1024), rel=1e-9)
    assert r.mfma_busy_pct == pytest.approx(59.815, abs=0.002)
    # SQ_WAVE_CYCLES (units of 4 cycles): (256398487 + 243068602) / 2 over 1024 SIMDs x 8 slots
    assert r.achieved_occupancy_pct == pytest.approx(100 * 4 * 249733544.5 / (wall * 1024 * 8), rel=1e-9)
    assert r.achieved_occupancy_pct == pytest.approx(20.706, abs=0.002)
    # SQ_LDS_BANK_CONFLICT 704512 of SQ_LDS_IDX_ACTIVE 35952128
    assert r.lds_bank_conflict_pct == pytest.approx(1.9596, abs=0.0002)
    # the counters replace the estimate: 60 % busy matrix pipes are not "MFMA-bound"
    assert r.bottleneck == tf.TF_BN_LATENCY
    assert tf.refine_hint(None, r, hw) == tf.TF_BN_LATENCY
    # a second file adds its fields and keeps the others
    tf.report_set_counters(r, hw, TCC_C3, "tf_gemm_lds_kernel")
    assert r.l2_hit_pct == pytest.approx(100 * 18754226.5 / (18754226.5 + 5613567.5), rel=1e-9)
    assert r.l2_hit_pct == pytest.approx(76.963, abs=0.002)
    assert r.mfma_busy_pct == pytest.approx(59.815, abs=0.002)
    # the other kernel in the same file (a register-only MFMA loop): 5242880000 busy cycles in 43250136 / 8 cycles
    r2 = blank_report()
    tf.report_set_counters(r2, hw, SQ_C3, "tf_calib_mfma_kernel")
    assert r2.mfma_busy_pct == pytest.approx(94.705, abs=0.002)
    assert r2.lds_bank_conflict_pct == 0.0
    assert r2.bottleneck == tf.TF_BN_MFMA


def test_memory_counters_are_scaled_and_timed_with_the_profiled_dispatches():
    hw = tf.hw_nominal()
    r = blank_report(t_med_us=50.0)
    tf.report_set_counters(r, hw, FETCH_C5, "tf_gemm_lds_kernel")
    # FETCH_SIZE (50240.625 + 49244.1875) / 2 KiB, priced at half the bytes -> x 2; dispatches of 48034 and 37475 ns
    assert r.hbm_read_gbs == pytest.approx(49742.40625 * 2 * 1024 / 42754.5, rel=1e-9)      # bytes per ns = GB/s
    assert r.hbm_read_gbs == pytest.approx(2382.7, abs=0.1)
    tf.report_set_counters(r, hw, WRITE_C5, "tf_gemm_lds_kernel")
    assert r.hbm_write_gbs == pytest.approx(16385.25 * 1024 / 41774.5, rel=1e-9)
    assert r.hbm_write_gbs == pytest.approx(401.64, abs=0.02)
    assert r.hbm_read_gbs == pytest.approx(2382.7, abs=0.1)
    # the reduce kernel of the same launches is told apart by its name
    r2 = blank_report()
    tf.report_set_counters(r2, hw, FETCH_C5, "tf_splitk_reduce_kernel")
    assert r2.hbm_read_gbs == pytest.approx((8227.5 + 8226.0) / 2 * 2 * 1024 / ((6599 + 6319) / 2), rel=1e-9)
    # a memory-bound report: the counters' traffic decides the class
    r3 = blank_report(arithmetic_intensity=15.9, pct_hbm_peak=10.0)
    assert tf.refine_hint(None, r3, hw) != tf.TF_BN_HBM
    r3.hbm_read_gbs, r3.hbm_write_gbs, r3.have_counters = 5000.0, 100.0, 1
    assert tf.refine_hint(None, r3, hw) == tf.TF_BN_HBM


def test_counter_file_errors(tmp_path):
    hw = tf.hw_nominal()
    r = blank_report()
    for path, sub in ((str(tmp_path / "missing.csv"), "tf_gemm"), (SQ_C3, "no_such_kernel")):
        with pytest.raises(tf.TfError) as e:
            tf.report_set_counters(r, hw, path, sub)
        assert e.value.status == tf.TF_E_PROFILER
    assert r.have_counters == 0
    bad = tmp_path / "nohdr.csv"
    bad.write_text('"Kernel","Value"\n"tf_gemm",1\n')
    with pytest.raises(tf.TfError) as e:
        tf.report_set_counters(r, hw, str(bad), "tf_gemm")
    assert e.value.status == tf.TF_E_PROFILER
    unknown = tmp_path / "unknown.csv"
    unknown.write_text('"Dispatch_Id","Kernel_Name","Counter_Name","Counter_Value"\n1,"tf_gemm<1, 2>","SOMETHING_ELSE",5\n')
    with pytest.raises(tf.TfError) as e:
        tf.report_set_counters(r, hw, str(unknown), "tf_gemm")
    assert e.value.status == tf.TF_E_PROFILER
    # a file without time stamps falls back on the report's own median for the rates; names with commas are one field
    plain = tmp_path / "plain.csv"
    plain.write_text('"Dispatch_Id","Kernel_Name","Counter_Name","Counter_Value"\n'
                     '1,"void k<LdsCfg<128, 128, 2, 4>, true>(P)","WRITE_SIZE",1000.0\n'
                     '2,"void k<LdsCfg<128, 128, 2, 4>, true>(P)","WRITE_SIZE",3000.0\n'
                     '3,"void k<LdsCfg<64, 64, 2, 2>, true>(P)","WRITE_SIZE",99999.0\n')
    r = blank_report(t_med_us=100.0)
    tf.report_set_counters(r, hw, str(plain), "LdsCfg<128, 128, 2, 4>")
    assert r.hbm_write_gbs == pytest.approx(2000.0 * 1024 / 100.0 * 1e-3, rel=1e-9)


LOOP_SQ_C3 = os.path.join(G, "rocprofv3_pmc_sq_loop_C3.csv")


def kernels_in(path):
    import csv
    with open(path, newline="") as f:
        return sorted({r["Kernel_Name"] for r in csv.DictReader(f)})


def test_kernel_name_of_a_variant_finds_its_rows_in_profiler_output():
    """rocprofv3_pmc_sq_loop_C3.csv: one dispatch each of five kernels from a profiler pass over the loop on
    4096 x 11008 x 4096. tf_variant_kernel_name must lead every variant to the rows of its own compiled kernel and
    to no other's."""
    kernels = kernels_in(LOOP_SQ_C3)
    assert len(kernels) == 5
    hw = tf.hw_nominal()
    with tf.Problem(4096, 11008, 4096) as p:
        vs = {v.name.decode(): v for v in p.variants()}
    expect = {
        "naive_1elem_per_thread": "tf_gemm_naive_kernel",
        "lds_256x256x64_w2x4_s2_direct_tail192_sk1x": "tf_gemm_mixed_kernel<tf::LdsCfg<256, 256, 64, 2, 4, 2, true, false, 1, false, false, 256>",
        "lds_256x256x64_w2x4_s2_direct_sk1": "tf_gemm_lds_kernel<tf::LdsCfg<256, 256, 64, 2, 4, 2, true, false, 1, false, false, 256>",
        "lds_256x256x32_w2x4_s4_direct_sk1x": "tf_gemm_lds_kernel<tf::LdsCfg<256, 256, 32, 2, 4, 4, true, false, 1, false, false, 256>",
        "lds_256x128x64_w4x2_s3_direct_sk1": "tf_gemm_lds_kernel<tf::LdsCfg<256, 128, 64, 4, 2, 3, true, false, 1, false, false, 128>",
    }
    for name, sub in expect.items():
        got = tf.kernel_substr(vs[name])
        assert got == sub
        hits = [k for k in kernels if got in k]
        assert len(hits) == 1, (name, hits)
        r = blank_report()
        tf.report_set_counters(r, hw, LOOP_SQ_C3, got)
        assert r.have_counters == 1 and r.achieved_occupancy_pct > 0
        assert (r.mfma_busy_pct == 0.0) == (name == "naive_1elem_per_thread")
    # the rotated K order is a run-time argument of the same kernel; a kernel that is not in the file is not found
    assert tf.kernel_substr(vs["lds_256x256x64_w2x4_s2_direct_sk1x"]) == tf.kernel_substr(vs["lds_256x256x64_w2x4_s2_direct_sk1"])
    other = tf.kernel_substr(vs["lds_128x128x64_w2x4_s3_direct_sk1"])
    assert not [k for k in kernels if other in k]
    with pytest.raises(tf.TfError):
        tf.report_set_counters(blank_report(), hw, LOOP_SQ_C3, other)
    # every variant of the family has a kernel name, and different compiled kernels have different names
    subs = {}
    for v in vs.values():
        s = tf.kernel_substr(v)
        assert s, v.name
        key = (v.kind, v.bm, v.bn, v.bk, v.waves_m, v.waves_n, v.waves_k, v.stages, v.direct_to_lds, v.a_bypass_lds, v.bn_tail > 0, v.stream_k)
        subs.setdefault(s, set()).add(key)
    assert all(len(k) == 1 for k in subs.values())
    # the large-tile kernel in steady state: 4096 MFMAs per SIMD and tile, 2.69 tiles per CU, hand-computed from the rows
    r = blank_report()
    tf.report_set_counters(r, hw, LOOP_SQ_C3, expect["lds_256x256x64_w2x4_s2_direct_tail192_sk1x"])
    assert 55.0 < r.mfma_busy_pct < 70.0 and 1.0 < r.lds_bank_conflict_pct < 3.0


def test_counter_files_handed_to_a_problem_are_checked():
    with tf.Problem(256, 256, 256) as p:
        p.set_counter_files([SQ_C3, TCC_C3])
        p.set_counter_files([])
        with pytest.raises(tf.TfError):
            p.set_counter_files([os.path.join(G, "no_such_file.csv")])
