#!/usr/bin/env python3
"""Benchmark of the tile kernel Y = GELU_erf(A.B + bias) on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C2] [--variant NAME] [--no-cpu]

One step = one launch of the kernel the variant loop selected, over one batch of synthetic
input that is already resident in HBM; batches rotate over enough buffer sets to exceed the
256 MB Infinity Cache, so operands are not served from cache left by the previous step.
The variant loop (Algorithm 1 of the paper: baseline profile, up to 8 rounds of proposal,
run, parity gate, profile, arbiter) runs once before the timed region; its result, its
round log and the tuned-vs-naive speedup are reported in the same JSON line.
Prints ONE JSON line on stdout; progress goes to stderr.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

BF16_PEAK_TFLOPS = 256 * 4096 * 2.4e9 / 1e12     # 2516.6: 256 CUs x 4096 flop/clk x 2.4 GHz, dense
HBM_PEAK_GBS = 8000.0
MALL_BYTES = 256 << 20


# rocprofv3 --pmc readings (KiB per dispatch) of the C2 kernels the loop ends on: (FETCH_SIZE, WRITE_SIZE).
# A 256 MiB device copy reads FETCH_SIZE 131086 and WRITE_SIZE 262144 KiB, hence the scale factors.
FETCH_SCALE, WRITE_SCALE = 262144.0 / 131084.9, 1.0
HBM_TRAFFIC_KIB = {
    ("C2", "lds_128x128x64_w2x4_s3_direct_sk1"): (24691.0, 8192.0),
    ("C2", "lds_128x128x64_w4x2_s3_direct_sk1"): (24690.6, 8192.0),
    ("C2", "lds_128x128x64_w2x4_s4_direct_sk1"): (24694.9, 8192.0),
    ("C2", "lds_128x128x64_w2x2x2_s3_direct_sk1"): (24690.5, 8192.0),
    ("C2", "lds_128x128x64_w2x2x2_s4_direct_sk1"): (24699.5, 8192.0),
    ("C2", "lds_128x128x64_w2x4_s3_direct_sk1x"): (24696.9, 8192.0),
    ("C2", "lds_128x128x64_w4x2_s3_direct_sk1x"): (24699.6, 8193.1),
    ("C2", "lds_128x128x64_w2x4_s4_direct_sk1x"): (24700.9, 8192.0),
    ("C2", "lds_128x128x64_w2x2x2_s3_direct_sk1x"): (24700.5, 8192.0),
    ("C2", "lds_128x128x64_w2x2x2_s4_direct_sk1x"): (24699.5, 8192.0),
    ("C3", "lds_256x256x64_w2x4_s2_direct_sk1"): (314016.0, 88064.9),
    ("C3", "lds_256x256x64_w4x2_s2_direct_sk1"): (303331.0, 88073.8),
    ("C3", "lds_256x256x64_w2x4_s2_direct_sk1x"): (309078.1, 88064.3),
    ("C3", "lds_256x256x64_w4x2_s2_direct_sk1x"): (303378.0, 88067.8),
    ("C4", "lds_32x64x64_w1x2_s4_direct_sk2l"): (67568.4, 1290.9),
    ("C4", "lds_32x64x64_w1x2_s4_direct_sk2r"): (66466.8 + 546.0, 1024.0 + 256.0),      # GEMM kernel + reduce kernel
    ("V2", "vecmat_r1_u4_w4_g0"): (525341.2, 1024.1),
    ("V2", "vecmat_r1_u8_w4_g0"): (525349.2, 1024.0),
    ("T2", "bgemm_128x128x64_w2x2_s2_ldstrans"): (16516.6, 131878.9),
    ("T2", "bgemm_128x128x64_w2x4_s2_ldstrans"): (16486.7, 131239.7),
    ("E2", "sin_b1024_t256_v4_g0_nt"): (131091.8, 262147.1),
    ("E2", "sin_b2048_t256_v4_g0_nt"): (131101.2, 262145.1),
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(w, A, B, bias, budget_s=12.0):
    """The oracle as it stands, single thread, on the first rows of the same workload."""
    from oracle import gemm_oracle as orc
    probe_rows = max(1, min(w.M, int(2e7 // max(1, w.N * w.K)) or 1))
    t0 = time.perf_counter()
    orc.gemm_bias_gelu(A[:probe_rows], B, bias)
    dt = time.perf_counter() - t0
    rows = int(max(probe_rows, min(w.M, probe_rows * budget_s / max(dt, 1e-6))))
    t0 = time.perf_counter()
    orc.gemm_bias_gelu(A[:rows], B, bias)
    dt = time.perf_counter() - t0
    flops = 2.0 * rows * w.N * w.K
    return {"value": flops / dt * 1e-12, "unit": "TFLOP/s", "cores": 1, "kind": "oracle",
            "sample": "first %d of %d rows of %s (%.2f GMAC) in %.2f s" % (rows, w.M, w.name, flops / 2e9, dt)}


def cpu_baseline_vecmat(w, A, B, budget_s=12.0):
    """The vector-matrix oracle as it stands, single thread, on the first matrices of the batch."""
    from oracle import gemm_oracle as orc
    t0 = time.perf_counter()
    orc.batched_vecmat(A[:1], B[:1])
    dt = time.perf_counter() - t0
    rows = int(max(1, min(w.M, budget_s / max(dt, 1e-6))))
    t0 = time.perf_counter()
    orc.batched_vecmat(A[:rows], B[:rows])
    dt = time.perf_counter() - t0
    flops = 2.0 * rows * w.N * w.K
    return {"value": flops / dt * 1e-12, "unit": "TFLOP/s", "cores": 1, "kind": "oracle",
            "sample": "first %d of %d matrices of %s (%.2f GMAC) in %.2f s" % (rows, w.M, w.name, flops / 2e9, dt)}


def cpu_baseline_bgemm(w, A, B, budget_s=12.0):
    """The batched transposed-operand oracle as it stands, single thread, on the first items of the batch."""
    from oracle import gemm_oracle as orc
    t0 = time.perf_counter()
    orc.batched_gemm_tn(A[:1, :, :64], B[:1])
    dt = (time.perf_counter() - t0) * w.M / 64.0
    items = int(max(1, min(w.batch, budget_s / max(dt, 1e-6))))
    t0 = time.perf_counter()
    orc.batched_gemm_tn(A[:items], B[:items])
    dt = time.perf_counter() - t0
    flops = 2.0 * items * w.M * w.N * w.K
    return {"value": flops / dt * 1e-12, "unit": "TFLOP/s", "cores": 1, "kind": "oracle",
            "sample": "first %d of %d items of %s (%.2f GMAC) in %.2f s" % (items, w.batch, w.name, flops / 2e9, dt)}


def cpu_baseline_sin(w, x, budget_s=12.0):
    """The sine oracle as it stands, single thread, on the first elements."""
    from oracle import gemm_oracle as orc
    t0 = time.perf_counter()
    orc.sin_f32(x[:1 << 20])
    dt = time.perf_counter() - t0
    n = int(max(1, min(w.n, (1 << 20) * budget_s / max(dt, 1e-6))))
    t0 = time.perf_counter()
    orc.sin_f32(x[:n])
    dt = time.perf_counter() - t0
    return {"value": n / dt * 1e-9, "unit": "Gelement/s", "cores": 1, "kind": "oracle",
            "sample": "first %d of %d elements of %s in %.2f s" % (n, w.n, w.name, dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # a timed region of tens of milliseconds: shorter ones read a few per cent low and scatter more (clock ramp)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="C2", choices=["C1", "C2", "C3", "C4", "C5", "V1", "V2", "T1", "T2", "E1", "E2"],
                    help="C1..C5: Y = GELU_erf(A.B + bias); V1, V2: batched vector-matrix product C[m,n] = sum_k A[m,k] B[m,n,k]; "
                         "T1, T2: batched transposed-operand product C[b] = A[b]^T B[b]; E1, E2: element-wise sine y = sin(x), fp32")
    ap.add_argument("--epilogue", default="gelu_erf", choices=["gelu_erf", "gelu_tanh", "bias"],
                    help="C1..C5 only: the bf16 epilogue (the headline metric is gelu_erf)")
    ap.add_argument("--variant", default=None, help="time this variant instead of the loop's choice")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-tune", action="store_true", help="skip the loop (needs --variant)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="launch a plain device copy of known size instead (reference reading for the HBM traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: the library runs on ONE GPU; --gpus %d is not supported (no collectives, no sharding)." % args.gpus)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2512_09196_amd import tf
    from paper_2512_09196_amd import workloads as wl

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible; there is no CPU path.")
        sys.exit(3)
    torch.cuda.set_device(0)
    if args.copy_calibration:
        # 256 MiB read + 256 MiB written per launch, from buffers that rotate past the memory-side cache
        n = 128 << 20
        src = [torch.ones(n, dtype=torch.int16, device="cuda") for _ in range(4)]
        dst = [torch.empty(n, dtype=torch.int16, device="cuda") for _ in range(4)]
        torch.cuda.synchronize()
        for i in range(args.warmup + args.steps):
            dst[i % 4].copy_(src[i % 4])
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": True, "launches": args.warmup + args.steps,
                          "bytes_read_per_launch": 2 * n, "bytes_written_per_launch": 2 * n}))
        return
    vecmat = args.workload.startswith("V")
    bgemm = args.workload.startswith("T")
    sin = args.workload.startswith("E")
    w = (wl.VECMAT_WORKLOADS[args.workload] if vecmat else wl.BGEMM_WORKLOADS[args.workload] if bgemm
         else wl.SIN_WORKLOADS[args.workload] if sin else wl.WORKLOADS[args.workload])
    if sin:
        log("generating %s (n=%d, seed %d)" % (w.name, w.n, w.seed))
        A = wl.make_sin_input(w.n, w.seed).view(np.int16)       # carried as raw 16-bit halves like the other operands
        B, bias = np.zeros(8, np.int16), None
    else:
        log("generating %s (M=%d N=%d K=%d, seed %d)" % (w.name, w.M, w.N, w.K, w.seed))
    if sin:
        pass
    elif vecmat:
        A, B = wl.make_vecmat(w.M, w.N, w.K, w.seed)
        bias = None
    elif bgemm:
        A, B = wl.make_bgemm(w.batch, w.M, w.N, w.K, w.seed)
        bias = None
    else:
        A, B, bias = wl.make_inputs(w)
    set_bytes = w.algorithmic_bytes
    nbuf = max(2, min(24, -(-2 * MALL_BYTES // set_bytes)))
    log("buffer sets: %d x %.1f MB" % (nbuf, set_bytes / 1e6))
    dA = [torch.from_numpy(A.view(np.int16)).cuda() for _ in range(nbuf)]
    dB = [torch.from_numpy(B.view(np.int16)).cuda() for _ in range(nbuf)]
    nobias = vecmat or bgemm or sin
    db = [None if nobias else torch.from_numpy(bias.view(np.int16)).cuda() for _ in range(nbuf)]
    yshape = (w.batch, w.M, w.N) if bgemm else (w.n,) if sin else (w.M, w.N)
    dY = [torch.empty(yshape, dtype=torch.float32 if nobias else torch.bfloat16, device="cuda") for _ in range(nbuf)]
    stream = torch.cuda.current_stream()
    bound_kind = "hbm" if nobias else w.bound      # T2: 179 flop/byte with the fp32 output counted, below the ridge

    if sin:
        prob = tf.Problem(1, w.n, 0, op=tf.TF_OP_ELEMENTWISE_SIN)
    elif bgemm:
        prob = tf.Problem(w.M, w.N, w.K, op=tf.TF_OP_BATCHED_GEMM_TN, batch=w.batch)
    else:
        epi = {"gelu_erf": tf.TF_EPI_BIAS_GELU_ERF, "gelu_tanh": tf.TF_EPI_BIAS_GELU_TANH, "bias": tf.TF_EPI_BIAS}[args.epilogue]
        prob = tf.Problem(w.M, w.N, w.K, op=tf.TF_OP_BATCHED_VECMAT if vecmat else tf.TF_OP_GEMM_EPILOGUE,
                          epi=tf.TF_EPI_NONE_F32 if vecmat else epi)
    variants = prob.variants()
    names = [v.name.decode() for v in variants]
    tune = None
    if not args.no_tune:
        t0 = time.perf_counter()
        best, rep, rlog = prob.tune(dA[0], dB[0], db[0], dY[0], stream=stream)
        tune_s = time.perf_counter() - t0
        rounds = [{"variant": names[r.variant_id], "t_med_us": round(r.t_med_us, 3), "status": r.status,
                   "parity_ok": r.parity_ok, "bottleneck": tf.BOTTLENECK_NAMES[r.bottleneck],
                   "pct_mfma_peak": round(r.pct_mfma_peak, 2), "pct_hbm_peak": round(r.pct_hbm_peak, 2)} for r in rlog]
        for r in rounds:
            log("  loop:", r)
        tune = {"selected": names[best], "rounds": len(rlog) - 1, "wall_s": round(tune_s, 3),
                "naive_us": round(rlog[0].t_med_us, 3), "tuned_us": round(rep.t_med_us, 3),
                "tuned_vs_naive": round(rlog[0].t_med_us / rep.t_med_us, 2),
                "one_shot_pick": rounds[1]["variant"] if len(rounds) > 1 else None,
                "one_shot_us": rounds[1]["t_med_us"] if len(rounds) > 1 else None, "log": rounds}
        vid = best
    if args.variant is not None:
        if args.variant not in names:
            log("unknown variant %s; have: %s" % (args.variant, ", ".join(names)))
            sys.exit(2)
        vid = names.index(args.variant)
    elif args.no_tune:
        log("--no-tune needs --variant")
        sys.exit(2)
    v = variants[vid]
    log("timing variant", names[vid])

    # marshal the arguments once: the timed loop is nothing but tf_variant_run calls
    import ctypes
    run = tf.lib().tf_variant_run
    sp = ctypes.c_void_p(stream.cuda_stream)
    argsets = [(prob._h, vid, ctypes.c_void_p(dA[j].data_ptr()), ctypes.c_void_p(dB[j].data_ptr()),
                None if nobias else ctypes.c_void_p(db[j].data_ptr()), ctypes.c_void_p(dY[j].data_ptr()), None, 0, sp)
               for j in range(nbuf)]
    prob.run(vid, dA[0], dB[0], db[0], dY[0], stream=stream)    # first use: workspace, attributes, errors raised

    def step(i):
        if run(*argsets[i % nbuf]) != 0:
            raise RuntimeError(tf.lib().tf_last_error().decode())

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    for i in range(args.steps):
        step(i)
    e1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ev_ms = e0.elapsed_time(e1)
    ms_per_step = wall_ms / args.steps
    kern_us = ev_ms * 1e3 / args.steps          # average launch duration on the launch stream
    tflops = w.flops / (ms_per_step * 1e-3) * 1e-12
    if bound_kind == "hbm":
        roof = {"bound": "hbm", "achieved": w.algorithmic_bytes / (kern_us * 1e-6) * 1e-9, "peak": HBM_PEAK_GBS,
                "unit": "GB/s"}
    else:
        roof = {"bound": "mfma", "achieved": w.flops / (kern_us * 1e-6) * 1e-12, "peak": BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    # HBM traffic per launch from the TCC counters (two rocprofv3 --pmc runs of this file with --variant),
    # scaled by what the same counters read for a plain 256 MiB copy; None for kernels not measured
    t = HBM_TRAFFIC_KIB.get((w.name, names[vid]))
    roof["traffic"] = None if t is None else (t[0] * FETCH_SCALE + t[1] * WRITE_SCALE) * 1024.0
    roof["traffic_unit"] = "bytes per launch"
    roof["kernel"] = names[vid]
    roof["avg_launch_us"] = kern_us
    # context: what this chip sustains right now on a register-only MFMA loop with data-like operands and on a
    # 1 GiB streaming read; `frac` stays the fraction of the published peak
    mfma_meas, hbm_meas = tf.hw_measure(0, stream)
    roof["measured_achievable"] = {"mfma_tflops": mfma_meas, "hbm_read_gbs": hbm_meas,
                                   "frac_of_measured": roof["achieved"] / (hbm_meas if bound_kind == "hbm" else mfma_meas)}

    if sin:
        workload = "%s: n=%d fp32, N(0, 10) inputs, seed %d" % (w.name, w.n, w.seed)
    else:
        workload = "%s: %sM=%d N=%d K=%d bf16, seed %d" % (w.name, "batch=%d " % w.batch if bgemm else "", w.M, w.N, w.K, w.seed)
    out = {
        "metric": ("element-wise sine Gelement/s (y = sin(x), fp32 in and out)" if sin else
                   "batched vector-matrix product TFLOP/s (C[m,n] = sum_k A[m,k] B[m,n,k], bf16 in, fp32 out)" if vecmat
                   else "batched transposed-operand product TFLOP/s (C[b] = A[b]^T B[b], bf16 in, fp32 out)" if bgemm
                   else "GEMM+epilogue TFLOP/s (bf16 %s, fp32 accumulate)"
                   % {"gelu_erf": "GELU_erf(A.B+bias)", "gelu_tanh": "GELU_tanh(A.B+bias)", "bias": "A.B+bias"}[args.epilogue]),
        "value": w.n / (ms_per_step * 1e-3) * 1e-9 if sin else tflops, "unit": "Gelement/s" if sin else "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if vecmat or sin else "bf16", "data": "synthetic",
        "config": {"workload": workload,
                   "variant": names[vid], "grid": v.grid, "split_k": v.split_k, "buffer_sets": nbuf},
        "pct_bf16_mfma_peak": 100.0 * tflops / BF16_PEAK_TFLOPS,
        "hbm_gbs_algorithmic": w.algorithmic_bytes / (ms_per_step * 1e-3) * 1e-9,
        "roofline": roof,
        "tune": tune,
    }
    if not args.no_cpu:
        log("timing the CPU oracle on a bounded sample ...")
        out["cpu_baseline"] = (cpu_baseline_sin(w, A.view(np.float32)) if sin else cpu_baseline_vecmat(w, A, B) if vecmat else cpu_baseline_bgemm(w, A, B) if bgemm
                               else cpu_baseline(w, A, B, bias))
    else:
        out["cpu_baseline"] = None
    prob.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
