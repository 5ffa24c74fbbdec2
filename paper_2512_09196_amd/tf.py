"""Thin ctypes binding over libtf_gfx950.so (declared in include/tf.h).

Argument marshalling only: every step of the hot path runs in the HIP kernels of the
library.  There is no fallback: if the library has not been built, loading raises.
Device buffers are passed as torch CUDA tensors (or raw integer addresses); torch is used
for device memory and streams only.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtf_gfx950.so")

TF_OK, TF_E_INVALID, TF_E_UNSUPPORTED, TF_E_LAUNCH, TF_E_NOMEM, TF_E_RANGE, TF_E_PROFILER = 0, -1, -2, -3, -4, -5, -6
TF_EPI_BIAS_GELU_ERF, TF_EPI_NONE_F32, TF_EPI_BIAS, TF_EPI_BIAS_GELU_TANH = 0, 1, 2, 3
TF_KIND_NAIVE, TF_KIND_MFMA_DIRECT, TF_KIND_MFMA_LDS, TF_KIND_MFMA_STREAM = 0, 1, 2, 3
TF_KIND_VECMAT_NAIVE, TF_KIND_VECMAT_STREAM, TF_KIND_BGEMM_TN_NAIVE, TF_KIND_SIN = 4, 5, 6, 7
TF_OP_GEMM_EPILOGUE, TF_OP_BATCHED_VECMAT, TF_OP_BATCHED_GEMM_TN, TF_OP_ELEMENTWISE_SIN = 0, 1, 2, 3
TF_BN_UNKNOWN, TF_BN_UNDERFILLED, TF_BN_HBM, TF_BN_MFMA, TF_BN_LDS_CONFLICT, TF_BN_OCCUPANCY, TF_BN_LATENCY = range(7)
TF_DEC_CONTINUE, TF_DEC_ACCEPT, TF_DEC_FINISH = 0, 1, 2
BOTTLENECK_NAMES = ["unknown", "underfilled", "hbm", "mfma", "lds_conflict", "occupancy", "latency"]


class _Struct(C.Structure):
    def as_dict(self):
        out = {}
        for name, _ in self._fields_:
            v = getattr(self, name)
            out[name] = v.decode() if isinstance(v, bytes) else v
        return out


class ProblemDesc(_Struct):
    _fields_ = [("M", C.c_int32), ("N", C.c_int32), ("K", C.c_int32),
                ("lda", C.c_int64), ("ldb", C.c_int64), ("ldy", C.c_int64),
                ("epi", C.c_int32), ("device", C.c_int32), ("op", C.c_int32), ("batch", C.c_int32),
                ("stride_a", C.c_int64), ("stride_b", C.c_int64), ("stride_y", C.c_int64), ("trans_b", C.c_int32)]


class VariantDesc(_Struct):
    _fields_ = [("id", C.c_int32), ("kind", C.c_int32), ("bm", C.c_int32), ("bn", C.c_int32), ("bk", C.c_int32),
                ("waves_m", C.c_int32), ("waves_n", C.c_int32), ("waves_k", C.c_int32), ("stages", C.c_int32), ("split_k", C.c_int32), ("fused_reduce", C.c_int32),
                ("direct_to_lds", C.c_int32), ("a_bypass_lds", C.c_int32), ("trans_a", C.c_int32), ("trans_b", C.c_int32), ("stream_k", C.c_int32), ("k_rotate", C.c_int32), ("persistent", C.c_int32), ("bn_tail", C.c_int32), ("nontemporal", C.c_int32), ("xcd_swizzle", C.c_int32), ("group_m", C.c_int32),
                ("threads", C.c_int32), ("lds_bytes", C.c_int32), ("grid", C.c_int32),
                ("workspace_bytes", C.c_int64), ("name", C.c_char * 64)]


class Report(_Struct):
    _fields_ = [("variant_id", C.c_int32), ("status", C.c_int32), ("warmup", C.c_int32), ("iters", C.c_int32),
                ("launches_per_iter", C.c_int32),
                ("t_min_us", C.c_double), ("t_med_us", C.c_double), ("t_mean_us", C.c_double), ("t_max_us", C.c_double),
                ("tflops", C.c_double), ("gbytes_per_s", C.c_double), ("pct_mfma_peak", C.c_double),
                ("pct_hbm_peak", C.c_double), ("arithmetic_intensity", C.c_double),
                ("grid", C.c_int32), ("waves_per_simd", C.c_int32),
                ("vgprs", C.c_int32), ("agprs", C.c_int32), ("sgprs", C.c_int32), ("spill_bytes", C.c_int32),
                ("lds_bytes", C.c_int32),
                ("occupancy_pct", C.c_double), ("grid_fill", C.c_double), ("have_counters", C.c_int32),
                ("mfma_busy_pct", C.c_double), ("lds_bank_conflict_pct", C.c_double), ("hbm_read_gbs", C.c_double),
                ("hbm_write_gbs", C.c_double), ("l2_hit_pct", C.c_double), ("achieved_occupancy_pct", C.c_double),
                ("bottleneck", C.c_int32), ("parity_ok", C.c_int32)]


class Hw(_Struct):
    _fields_ = [("name", C.c_char * 64), ("cus", C.c_int32), ("simds_per_cu", C.c_int32), ("wave_size", C.c_int32),
                ("xcds", C.c_int32), ("lds_bytes_per_cu", C.c_int32), ("vgprs_per_simd_lane", C.c_int32),
                ("max_waves_per_simd", C.c_int32), ("l2_bytes", C.c_int64), ("hbm_bytes", C.c_int64),
                ("clock_mhz", C.c_double), ("hbm_gbs_peak", C.c_double), ("bf16_tflops_peak", C.c_double)]


class Theta(_Struct):
    _fields_ = [("first_accept_speedup", C.c_double), ("later_accept_gain", C.c_double),
                ("robust_spread", C.c_double), ("patience", C.c_int32), ("max_rounds", C.c_int32),
                ("cold_bytes", C.c_int64)]


PARITY_FN = C.CFUNCTYPE(C.c_int32, C.c_void_p, C.c_int32)

# name -> (restype, argtypes): every function include/tf.h declares
_P = C.POINTER
SIGNATURES = {
    "tf_theta_default": (None, [_P(Theta)]),
    "tf_hw_query": (C.c_int32, [C.c_int32, _P(Hw)]),
    "tf_hw_nominal": (None, [_P(Hw)]),
    "tf_hw_measure": (C.c_int32, [C.c_int32, C.c_void_p, _P(C.c_double), _P(C.c_double)]),
    "tf_hw_read_rate": (C.c_int32, [C.c_int32, C.c_void_p, _P(C.c_void_p), C.c_int32, C.c_int64, C.c_int32, _P(C.c_double)]),
    "tf_problem_create": (C.c_int32, [_P(ProblemDesc), _P(C.c_void_p)]),
    "tf_problem_destroy": (None, [C.c_void_p]),
    "tf_variant_enumerate": (C.c_int32, [C.c_void_p, _P(VariantDesc), C.c_int32]),
    "tf_variant_run": (C.c_int32, [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                   C.c_void_p, C.c_size_t, C.c_void_p]),
    "tf_variant_profile": (C.c_int32, [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_size_t, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                       _P(Report)]),
    "tf_variant_run_static": (C.c_int32, [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.c_void_p]),
    "tf_static_scratch_bytes": (C.c_int64, []),
    "tf_workspace_status": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "tf_xcc_placement_ok": (C.c_int32, [_P(C.c_uint32), C.c_int32]),
    "tf_gate_count_bad": (C.c_int64, [C.c_void_p, C.c_int64, _P(C.c_float), _P(C.c_float), _P(C.c_float), C.c_int64,
                                      C.c_int32, C.c_int32, C.c_int32, C.c_int32]),
    "tf_report_set_counters": (C.c_int32, [_P(Report), _P(Hw), C.c_char_p, C.c_char_p]),
    "tf_variant_kernel_name": (C.c_int32, [_P(VariantDesc), C.c_char_p, C.c_int32]),
    "tf_problem_set_counter_files": (C.c_int32, [C.c_void_p, _P(C.c_char_p), C.c_int32]),
    "tf_arbiter": (C.c_int32, [_P(Report), _P(Report), _P(Theta), C.c_int32, C.c_int32, C.c_int32]),
    "tf_refine_hint": (C.c_int32, [_P(Report), _P(Report), _P(Hw)]),
    "tf_proposal": (C.c_int32, [_P(ProblemDesc), _P(Hw), _P(VariantDesc), C.c_int32, _P(C.c_uint8), C.c_int32,
                                C.c_int32]),
    "tf_proposal_from": (C.c_int32, [_P(Hw), _P(VariantDesc), _P(C.c_double), C.c_int32, _P(C.c_uint8), C.c_int32,
                                     C.c_int32]),
    "tf_predict_us": (C.c_double, [_P(ProblemDesc), _P(Hw), _P(VariantDesc)]),
    "tf_resident_wgs": (C.c_int32, [_P(Hw), _P(VariantDesc)]),
    "tf_grid_fill": (C.c_double, [_P(Hw), _P(VariantDesc)]),
    "tf_tune_replay": (C.c_int32, [_P(ProblemDesc), _P(Hw), _P(VariantDesc), _P(Report), C.c_int32, _P(Theta),
                                   _P(C.c_int32), _P(Report), _P(Report), C.c_int32, _P(C.c_int32)]),
    "tf_tune": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                            C.c_void_p, _P(Theta), PARITY_FN, C.c_void_p, _P(C.c_int32), _P(Report), _P(Report),
                            C.c_int32, _P(C.c_int32)]),
    "tf_last_error": (C.c_char_p, []),
    "tf_version": (C.c_char_p, []),
    "tf_struct_sizes": (None, [_P(C.c_int32)]),
}

_lib = None


class TfError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__("tf status %d: %s" % (status, msg))
        self.status = status


def lib():
    """The loaded library. Raises if it has not been built: there is no other code path."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "%s is missing: build it with `python -m paper_2512_09196_amd.build` "
                "(the HIP library is the only implementation)" % LIB_PATH)
        # PyTorch ships its own HIP runtime. If it is going to be used in this process (device memory,
        # streams), it must be loaded first, so that this library binds to the same runtime instance
        # instead of bringing in a second one that does not see the first one's device state.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            f = getattr(l, name)
            f.restype = res
            f.argtypes = args
        built = (C.c_int32 * 5)()
        l.tf_struct_sizes(built)
        mine = [C.sizeof(t) for t in (ProblemDesc, VariantDesc, Report, Hw, Theta)]
        if list(built) != mine:
            raise RuntimeError("%s was built from another include/tf.h (struct sizes %s, this binding has %s): "
                               "rebuild it with `python -m paper_2512_09196_amd.build`" % (LIB_PATH, list(built), mine))
        _lib = l
    return _lib


def _check(st):
    if st != TF_OK:
        raise TfError(st, lib().tf_last_error().decode())


def _ptr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return C.c_void_p(x)
    return C.c_void_p(x.data_ptr())   # torch tensor


def _stream(stream):
    if stream is None:
        import torch
        return C.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return C.c_void_p(stream)
    return C.c_void_p(stream.cuda_stream)


def theta_default() -> Theta:
    t = Theta()
    lib().tf_theta_default(C.byref(t))
    return t


def hw_nominal() -> Hw:
    h = Hw()
    lib().tf_hw_nominal(C.byref(h))
    return h


def hw_query(device: int = 0) -> Hw:
    h = Hw()
    _check(lib().tf_hw_query(device, C.byref(h)))
    return h


def hw_measure(device: int = 0, stream=None):
    """(bf16 MFMA TFLOP/s of a register-only loop, GB/s of a 1 GiB streaming read), measured now."""
    a, b = C.c_double(0.0), C.c_double(0.0)
    _check(lib().tf_hw_measure(device, _stream(stream), C.byref(a), C.byref(b)))
    return a.value, b.value


def hw_read_rate(buffers, nbytes: int, launches: int, device: int = 0, stream=None) -> float:
    """GB/s of a plain streaming read of nbytes per launch, rotating over the given device tensors."""
    arr = (C.c_void_p * len(buffers))(*[b.data_ptr() for b in buffers])
    g = C.c_double(0.0)
    _check(lib().tf_hw_read_rate(device, _stream(stream), arr, len(buffers), nbytes, launches, C.byref(g)))
    return g.value


def arbiter(cand: Report, best: Report, theta: Theta, best_is_baseline: bool, stall_rounds: int, rnd: int) -> int:
    return lib().tf_arbiter(C.byref(cand), C.byref(best), C.byref(theta), int(best_is_baseline), stall_rounds, rnd)


def refine_hint(prev, cand: Report, hw: Hw) -> int:
    return lib().tf_refine_hint(C.byref(prev) if prev is not None else None, C.byref(cand), C.byref(hw))


def predict_us(desc: ProblemDesc, hw: Hw, v: VariantDesc) -> float:
    return lib().tf_predict_us(C.byref(desc), C.byref(hw), C.byref(v))


def resident_wgs(hw: Hw, v: VariantDesc) -> int:
    return lib().tf_resident_wgs(C.byref(hw), C.byref(v))


def grid_fill(hw: Hw, v: VariantDesc) -> float:
    return lib().tf_grid_fill(C.byref(hw), C.byref(v))


def _array(cls, items):
    arr = (cls * len(items))()
    for i, it in enumerate(items):
        C.memmove(C.byref(arr[i]), C.byref(it), C.sizeof(cls))
    return arr


def proposal_from(hw: Hw, family, predicted, tried, base_id: int, bottleneck: int) -> int:
    fam = _array(VariantDesc, family)
    pred = (C.c_double * len(family))(*predicted)
    tr = (C.c_uint8 * len(family))(*[1 if t else 0 for t in tried])
    return lib().tf_proposal_from(C.byref(hw), fam, pred, len(family), tr, base_id, bottleneck)


def proposal(desc: ProblemDesc, hw: Hw, family, tried, base_id: int, bottleneck: int) -> int:
    fam = _array(VariantDesc, family)
    tr = (C.c_uint8 * len(family))(*[1 if t else 0 for t in tried])
    return lib().tf_proposal(C.byref(desc), C.byref(hw), fam, len(family), tr, base_id, bottleneck)


def tune_replay(desc: ProblemDesc, hw: Hw, family, reports, theta: Theta):
    """Algorithm 1 over pre-made reports. Returns (best_variant, best_report, [round reports])."""
    fam = _array(VariantDesc, family)
    rep = _array(Report, reports)
    cap = 1 + theta.max_rounds
    log = (Report * cap)()
    best = Report()
    bv = C.c_int32(-1)
    nl = C.c_int32(0)
    _check(lib().tf_tune_replay(C.byref(desc), C.byref(hw), fam, rep, len(family), C.byref(theta),
                                C.byref(bv), C.byref(best), log, cap, C.byref(nl)))
    return bv.value, best, [log[i] for i in range(nl.value)]


def xcc_placement_ok(xcc_of_wg) -> bool:
    arr = (C.c_uint32 * len(xcc_of_wg))(*[int(x) for x in xcc_of_wg])
    return bool(lib().tf_xcc_placement_ok(arr, len(xcc_of_wg)))


def gate_count_bad(Y, zref, norm_a, norm_b, K: int, epi: int, norm_b_row_stride: int = 0) -> int:
    """tf_tune's built-in comparison on host arrays (numpy): Y uint16 bf16 bits or float32 [rows, N] (C-contiguous
    rows; ldy = its row stride), zref float32 [rows, N] dense, norms float32. Returns the number of rejected elements."""
    import numpy as np
    rows, N = zref.shape
    zref = np.ascontiguousarray(zref, dtype=np.float32)
    norm_a = np.ascontiguousarray(norm_a, dtype=np.float32)
    norm_b = np.ascontiguousarray(norm_b, dtype=np.float32)
    assert Y.dtype == (np.float32 if epi == TF_EPI_NONE_F32 else np.uint16) and Y.shape[0] == rows and Y.strides[1] == Y.itemsize
    ldy = Y.strides[0] // Y.itemsize
    fp = lambda a: a.ctypes.data_as(_P(C.c_float))
    r = lib().tf_gate_count_bad(C.c_void_p(Y.ctypes.data), ldy, fp(zref), fp(norm_a), fp(norm_b), norm_b_row_stride, rows, N, K, epi)
    if r < 0:
        _check(int(r))
    return int(r)


def kernel_substr(v: VariantDesc):
    """The part of the kernel's name in a profiler's output that identifies the compiled kernel behind variant v
    (variants that differ only in launch parameters, such as K slices or the K order, share a kernel), or None."""
    buf = C.create_string_buffer(256)
    n = lib().tf_variant_kernel_name(C.byref(v), buf, 256)
    if n < 0:
        _check(int(n))
    return buf.value.decode() if n > 0 else None


def report_set_counters(report: Report, hw: Hw, csv_path: str, kernel_substr: str) -> None:
    _check(lib().tf_report_set_counters(C.byref(report), C.byref(hw), csv_path.encode(), kernel_substr.encode()))


class Problem:
    """tf_problem handle: one (M, N, K, strides, epilogue) instance of the tile kernel."""

    def __init__(self, M, N, K, lda=None, ldb=None, ldy=None, epi=TF_EPI_BIAS_GELU_ERF, device=0,
                 op=TF_OP_GEMM_EPILOGUE, batch=1, stride_a=None, stride_b=None, stride_y=None, trans_b=0):
        lda_default, ldb_default = K, (K if trans_b else N)
        if op == TF_OP_BATCHED_VECMAT:
            # C[m, n] = sum_k A[m, k] B[m, n, k]: B rows are K long, the output is fp32
            ldb_default, epi = K, TF_EPI_NONE_F32
        elif op == TF_OP_ELEMENTWISE_SIN:
            # Y[i] = sin(A[i]), i < N: fp32 in and out
            epi = TF_EPI_NONE_F32
        elif op == TF_OP_BATCHED_GEMM_TN:
            # C[b, m, n] = sum_k A[b, k, m] B[b, k, n]: A rows are M long, the output is fp32
            lda_default, epi = M, TF_EPI_NONE_F32
        lda = lda_default if lda is None else lda
        ldb = ldb_default if ldb is None else ldb
        ldy = N if ldy is None else ldy
        self.desc = ProblemDesc(M, N, K, lda, ldb, ldy, epi, device, op, batch,
                                K * lda if stride_a is None else stride_a, K * ldb if stride_b is None else stride_b,
                                M * ldy if stride_y is None else stride_y, 1 if trans_b else 0)
        self._h = C.c_void_p()
        _check(lib().tf_problem_create(C.byref(self.desc), C.byref(self._h)))

    def close(self):
        if self._h:
            lib().tf_problem_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    def variants(self):
        n = lib().tf_variant_enumerate(self._h, None, 0)
        if n < 0:
            _check(n)
        arr = (VariantDesc * n)()
        n2 = lib().tf_variant_enumerate(self._h, arr, n)
        if n2 < 0:
            _check(n2)
        return [arr[i] for i in range(n2)]

    def run(self, variant_id, A, B, bias, Y, workspace=None, workspace_bytes=0, stream=None):
        _check(lib().tf_variant_run(self._h, variant_id, _ptr(A), _ptr(B), _ptr(bias), _ptr(Y), _ptr(workspace),
                                    workspace_bytes, _stream(stream)))

    def run_static(self, variant_id, A, B, bias, Y, stream=None):
        """tf_variant_run on the workspace that is part of the library's device image: allocates nothing."""
        _check(lib().tf_variant_run_static(self._h, variant_id, _ptr(A), _ptr(B), _ptr(bias), _ptr(Y), _stream(stream)))

    def set_counter_files(self, paths):
        """Profiler counter CSVs of earlier passes: tune() then attaches them to every round's report before the hint."""
        arr = (C.c_char_p * max(1, len(paths)))(*[p.encode() for p in paths])
        _check(lib().tf_problem_set_counter_files(self._h, arr, len(paths)))

    def workspace_status(self, workspace=None, stream=None):
        """Synchronises the stream; raises TfError(TF_E_LAUNCH) if an L2-local reduction reported a misplaced slice."""
        _check(lib().tf_workspace_status(self._h, _ptr(workspace), _stream(stream)))

    def profile(self, variant_id, A, B, bias, Y, workspace=None, workspace_bytes=0, stream=None,
                warmup=3, iters=5, launches_per_iter=0) -> Report:
        r = Report()
        _check(lib().tf_variant_profile(self._h, variant_id, _ptr(A), _ptr(B), _ptr(bias), _ptr(Y), _ptr(workspace),
                                        workspace_bytes, _stream(stream), warmup, iters, launches_per_iter,
                                        C.byref(r)))
        return r

    def tune(self, A, B, bias, Y, workspace=None, workspace_bytes=0, stream=None, theta=None, parity=None):
        """Algorithm 1 on the GPU. parity: optional callable(variant_id) -> bool called after each
        BuildRun with Y holding that variant's output; by default the library compares every
        candidate with the baseline kernel's output. Returns (best_variant, best_report, log)."""
        th = theta if theta is not None else theta_default()
        cap = 1 + th.max_rounds
        log = (Report * cap)()
        best = Report()
        bv = C.c_int32(-1)
        nl = C.c_int32(0)
        cb = PARITY_FN(lambda user, vid: 1 if parity(vid) else 0) if parity is not None else PARITY_FN()
        _check(lib().tf_tune(self._h, _ptr(A), _ptr(B), _ptr(bias), _ptr(Y), _ptr(workspace), workspace_bytes,
                             _stream(stream), C.byref(th), cb, None, C.byref(bv), C.byref(best), log, cap,
                             C.byref(nl)))
        return bv.value, best, [log[i] for i in range(nl.value)]
