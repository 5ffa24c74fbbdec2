"""ctypes front end of the C oracle in ``tf_oracle.c``.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's cpu_baseline leg, never by the product package.  It builds the C
file with gcc (no fast-math, no vectorisation flags beyond -O2) into
``oracle/libtf_oracle.so`` and marshals numpy arrays; it holds no arithmetic.

The operation is  Y = GELU_erf(A.B + bias)  on bf16 bit patterns (numpy uint16),
evaluated in double; see the header of ``tf_oracle.c`` for the definition and
for what pins it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tf_oracle.c")
_LIB = os.path.join(_HERE, "libtf_oracle.so")
_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile tf_oracle.c -> libtf_oracle.so (skipped when up to date)."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    tmp = _LIB + ".tmp.%d" % os.getpid()
    cmd = ["gcc", "-std=c11", "-O2", "-fPIC", "-shared", "-fno-fast-math",
           "-ffp-contract=off", "-o", tmp, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build())
            u16p = ctypes.POINTER(ctypes.c_uint16)
            f64p = ctypes.POINTER(ctypes.c_double)
            i32p = ctypes.POINTER(ctypes.c_int)
            lib.tfo_bf16_to_double.restype = ctypes.c_double
            lib.tfo_bf16_to_double.argtypes = [ctypes.c_uint16]
            lib.tfo_gelu.restype = ctypes.c_double
            lib.tfo_gelu.argtypes = [ctypes.c_double]
            lib.tfo_gelu_tanh.restype = ctypes.c_double
            lib.tfo_gelu_tanh.argtypes = [ctypes.c_double]
            lib.tfo_gelu_tanh_array.restype = ctypes.c_int
            lib.tfo_gelu_tanh_array.argtypes = [ctypes.c_long, f64p, f64p]
            lib.tfo_gemm_bias_gelu.restype = ctypes.c_int
            lib.tfo_gemm_bias_gelu.argtypes = [
                ctypes.c_int, ctypes.c_int, ctypes.c_int, u16p, ctypes.c_long,
                u16p, ctypes.c_long, u16p, f64p, f64p, f64p]
            lib.tfo_gemm_nt_bias_gelu.restype = ctypes.c_int
            lib.tfo_gemm_nt_bias_gelu.argtypes = [
                ctypes.c_int, ctypes.c_int, ctypes.c_int, u16p, ctypes.c_long,
                u16p, ctypes.c_long, u16p, f64p, f64p, f64p]
            lib.tfo_batched_vecmat.restype = ctypes.c_int
            lib.tfo_batched_vecmat.argtypes = [
                ctypes.c_int, ctypes.c_int, ctypes.c_int, u16p, ctypes.c_long,
                u16p, ctypes.c_long, f64p, f64p]
            lib.tfo_batched_gemm_tn.restype = ctypes.c_int
            lib.tfo_batched_gemm_tn.argtypes = [
                ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, u16p, ctypes.c_long, ctypes.c_long,
                u16p, ctypes.c_long, ctypes.c_long, f64p, f64p]
            lib.tfo_sin_f32.restype = ctypes.c_int
            lib.tfo_sin_f32.argtypes = [ctypes.c_long, ctypes.POINTER(ctypes.c_float), f64p]
            lib.tfo_gemm_bias_gelu_at.restype = ctypes.c_int
            lib.tfo_gemm_bias_gelu_at.argtypes = [
                ctypes.c_int, ctypes.c_int, ctypes.c_int, u16p, ctypes.c_long,
                u16p, ctypes.c_long, u16p, ctypes.c_long, i32p, i32p,
                f64p, f64p, f64p]
            _lib = lib
    return _lib


def _u16(a, name):
    a = np.asarray(a)
    if a.dtype != np.uint16:
        raise TypeError(f"{name} must hold bf16 bit patterns as uint16, got {a.dtype}")
    return np.ascontiguousarray(a)


def _ptr(a, ty):
    return a.ctypes.data_as(ctypes.POINTER(ty))


def bf16_to_double(bits: int) -> float:
    return float(_load().tfo_bf16_to_double(int(bits) & 0xFFFF))


def gelu(z: float) -> float:
    return float(_load().tfo_gelu(float(z)))


def gelu_tanh(z):
    """The tanh form of GELU, 1/2 z (1 + tanh(sqrt(2/pi) (z + 0.044715 z^3))), of a float or a float64 array."""
    if np.isscalar(z):
        return float(_load().tfo_gelu_tanh(float(z)))
    z = np.ascontiguousarray(z, dtype=np.float64)
    y = np.empty_like(z)
    rc = _load().tfo_gelu_tanh_array(z.size, _ptr(z, ctypes.c_double), _ptr(y, ctypes.c_double))
    if rc != 0:
        raise RuntimeError(f"tfo_gelu_tanh_array failed with {rc}")
    return y


def gemm_bias_gelu(A, B, bias):
    """A: uint16 [M,K], B: uint16 [K,N], bias: uint16 [N].

    Returns (y, z, s): float64 [M,N] arrays -- the activation, the
    pre-activation and the absolute-value sum used by error bounds.
    """
    A, B, bias = _u16(A, "A"), _u16(B, "B"), _u16(bias, "bias")
    if A.ndim != 2 or B.ndim != 2 or bias.ndim != 1:
        raise ValueError("A and B must be 2-D, bias 1-D")
    M, K = A.shape
    K2, N = B.shape
    if K2 != K or bias.shape[0] != N:
        raise ValueError(f"shape mismatch A{A.shape} B{B.shape} bias{bias.shape}")
    y = np.empty((M, N), np.float64)
    z = np.empty((M, N), np.float64)
    s = np.empty((M, N), np.float64)
    rc = _load().tfo_gemm_bias_gelu(
        M, N, K, _ptr(A, ctypes.c_uint16), K,
        _ptr(B, ctypes.c_uint16), N,
        _ptr(bias, ctypes.c_uint16),
        _ptr(y, ctypes.c_double), _ptr(z, ctypes.c_double), _ptr(s, ctypes.c_double))
    if rc != 0:
        raise RuntimeError(f"tfo_gemm_bias_gelu failed with {rc}")
    return y, z, s


def gemm_nt_bias_gelu(A, Bt, bias):
    """The same operation with the second operand given as [N, K] (k contiguous): z = A . Bt^T + bias.

    A: uint16 [M, K], Bt: uint16 [N, K], bias: uint16 [N]. Returns (y, z, s), float64 [M, N]."""
    A, Bt, bias = _u16(A, "A"), _u16(Bt, "Bt"), _u16(bias, "bias")
    if A.ndim != 2 or Bt.ndim != 2 or bias.ndim != 1:
        raise ValueError("A and Bt must be 2-D, bias 1-D")
    M, K = A.shape
    N, K2 = Bt.shape
    if K2 != K or bias.shape[0] != N:
        raise ValueError(f"shape mismatch A{A.shape} Bt{Bt.shape} bias{bias.shape}")
    y = np.empty((M, N), np.float64)
    z = np.empty((M, N), np.float64)
    s = np.empty((M, N), np.float64)
    rc = _load().tfo_gemm_nt_bias_gelu(
        M, N, K, _ptr(A, ctypes.c_uint16), K, _ptr(Bt, ctypes.c_uint16), K, _ptr(bias, ctypes.c_uint16),
        _ptr(y, ctypes.c_double), _ptr(z, ctypes.c_double), _ptr(s, ctypes.c_double))
    if rc != 0:
        raise RuntimeError(f"tfo_gemm_nt_bias_gelu failed with {rc}")
    return y, z, s


def gemm_bias_gelu_at(A, B, bias, rows, cols):
    """The same three quantities at the listed (row, col) positions only."""
    A, B, bias = _u16(A, "A"), _u16(B, "B"), _u16(bias, "bias")
    M, K = A.shape
    K2, N = B.shape
    if K2 != K or bias.shape[0] != N:
        raise ValueError(f"shape mismatch A{A.shape} B{B.shape} bias{bias.shape}")
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    cols = np.ascontiguousarray(cols, dtype=np.int32)
    if rows.shape != cols.shape or rows.ndim != 1:
        raise ValueError("rows and cols must be 1-D and of equal length")
    n = rows.shape[0]
    y = np.empty(n, np.float64)
    z = np.empty(n, np.float64)
    s = np.empty(n, np.float64)
    rc = _load().tfo_gemm_bias_gelu_at(
        M, N, K, _ptr(A, ctypes.c_uint16), K, _ptr(B, ctypes.c_uint16), N,
        _ptr(bias, ctypes.c_uint16), n, _ptr(rows, ctypes.c_int), _ptr(cols, ctypes.c_int),
        _ptr(y, ctypes.c_double), _ptr(z, ctypes.c_double), _ptr(s, ctypes.c_double))
    if rc != 0:
        raise RuntimeError(f"tfo_gemm_bias_gelu_at failed with {rc}")
    return y, z, s


def batched_vecmat(A, B):
    """C[m, n] = sum_k A[m, k] B[m, n, k] (the paper's Case Study 2) in double, and S = sum |a b|.

    A: uint16 [M, K], B: uint16 [M, N, K], bf16 bit patterns. Returns (C, S), float64 [M, N]."""
    A, B = _u16(A, "A"), _u16(B, "B")
    if A.ndim != 2 or B.ndim != 3 or B.shape[0] != A.shape[0] or B.shape[2] != A.shape[1]:
        raise ValueError(f"shape mismatch A{A.shape} B{B.shape}")
    M, K = A.shape
    N = B.shape[1]
    c = np.empty((M, N), np.float64)
    s = np.empty((M, N), np.float64)
    rc = _load().tfo_batched_vecmat(M, N, K, _ptr(A, ctypes.c_uint16), K, _ptr(B, ctypes.c_uint16), K,
                                    _ptr(c, ctypes.c_double), _ptr(s, ctypes.c_double))
    if rc != 0:
        raise RuntimeError(f"tfo_batched_vecmat failed with {rc}")
    return c, s


def batched_gemm_tn(A, B):
    """C[b, m, n] = sum_k A[b, k, m] B[b, k, n] (the paper's Case Study 3, dB = dO^T A) in double, and S = sum |a b|.

    A: uint16 [batch, K, M], B: uint16 [batch, K, N], bf16 bit patterns. Returns (C, S), float64 [batch, M, N]."""
    A, B = _u16(A, "A"), _u16(B, "B")
    if A.ndim != 3 or B.ndim != 3 or A.shape[0] != B.shape[0] or A.shape[1] != B.shape[1]:
        raise ValueError(f"shape mismatch A{A.shape} B{B.shape}")
    batch, K, M = A.shape
    N = B.shape[2]
    c = np.empty((batch, M, N), np.float64)
    s = np.empty((batch, M, N), np.float64)
    rc = _load().tfo_batched_gemm_tn(batch, M, N, K, _ptr(A, ctypes.c_uint16), M, K * M,
                                     _ptr(B, ctypes.c_uint16), N, K * N,
                                     _ptr(c, ctypes.c_double), _ptr(s, ctypes.c_double))
    if rc != 0:
        raise RuntimeError(f"tfo_batched_gemm_tn failed with {rc}")
    return c, s


def sin_f32(x):
    """y = sin(x) in double for binary32 inputs (the paper's Case Study 1). x: float32 array; returns float64."""
    x = np.ascontiguousarray(x)
    if x.dtype != np.float32 or x.ndim != 1:
        raise ValueError("x must be a 1-D float32 array")
    y = np.empty(x.shape[0], np.float64)
    rc = _load().tfo_sin_f32(x.shape[0], _ptr(x, ctypes.c_float), _ptr(y, ctypes.c_double))
    if rc != 0:
        raise RuntimeError(f"tfo_sin_f32 failed with {rc}")
    return y
