"""Seeded synthetic inputs for the GEMM + bias + GELU tile kernel.

This module only draws numbers: it contains none of the kernel's arithmetic and
is the single piece of code that both the GPU path's tests and the CPU oracle's
tests use, so that both see the same bf16 bit patterns.

Generator (counter based, order independent, identical on every host):
  key   = seed * 2**40  XOR  tensor_id * 2**36
  u(i)  = top 53 bits of splitmix64(key XOR i) / 2**53            in [0, 1)
  uniform[-1,1) * scale :  (2 u(i) - 1) * scale
  normal(0, sigma)      :  Box-Muller on the pair u(2i), u(2i+1):
                           sigma * sqrt(-2 ln(1 - u(2i))) * cos(2 pi u(2i+1))
Values are computed in float64 and rounded once, round-to-nearest-even, to
bf16; tensors are returned as numpy uint16 bit patterns.

The five workloads (tensor ids: A = 0, B = 1, bias = 2; "sigma" is a standard
deviation; workload i uses seed i - 1):
  C1  M=N=K=256            A, B uniform[-1,1)/sqrt(K)   bias N(0,1)      seed 0
  C2  M=N=K=2048           same distributions                           seed 1
  C3  M=4096 K=4096 N=11008  A N(0,1)  B N(0,0.02)  bias N(0,0.01)      seed 2
  C4  M=16 K=8192 N=8192     A N(0,1)  B N(0,0.02)  bias N(0,0.01)      seed 3
  C5  M=N=1024 K=16384     A, B uniform[-1,1)/sqrt(K)   bias N(0,1)      seed 4
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

_MASK64 = np.uint64(0xFFFFFFFFFFFFFFFF)
_CHUNK = 1 << 22


def _splitmix64(x: np.ndarray) -> np.ndarray:
    """One step of the splitmix64 output function on uint64 counters."""
    with np.errstate(over="ignore"):
        z = x + np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


def _key(seed: int, tensor_id: int) -> np.uint64:
    return np.uint64(((int(seed) << 40) ^ (int(tensor_id) << 36)) & 0xFFFFFFFFFFFFFFFF)


def unit_uniform(seed: int, tensor_id: int, start: int, count: int) -> np.ndarray:
    """u(i) for i in [start, start+count): float64 in [0, 1)."""
    idx = np.arange(start, start + count, dtype=np.uint64)
    bits = _splitmix64(idx ^ _key(seed, tensor_id))
    return (bits >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def f64_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float64 -> float32 -> bf16, nearest-even, return uint16 bit patterns.

    The double rounding f64 -> f32 -> bf16 is part of the generator's
    definition; the result is the tensor, whatever value it approximates.
    """
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    w = f.view(np.uint32)
    lsb = (w >> np.uint32(16)) & np.uint32(1)
    r = (w + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to float32 (exact)."""
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def uniform_bf16(seed: int, tensor_id: int, shape, scale: float) -> np.ndarray:
    n = int(np.prod(shape))
    out = np.empty(n, np.uint16)
    for s in range(0, n, _CHUNK):
        c = min(_CHUNK, n - s)
        u = unit_uniform(seed, tensor_id, s, c)
        out[s:s + c] = f64_to_bf16_bits((2.0 * u - 1.0) * scale)
    return out.reshape(shape)


def normal_bf16(seed: int, tensor_id: int, shape, sigma: float, mean: float = 0.0) -> np.ndarray:
    n = int(np.prod(shape))
    out = np.empty(n, np.uint16)
    for s in range(0, n, _CHUNK):
        c = min(_CHUNK, n - s)
        u = unit_uniform(seed, tensor_id, 2 * s, 2 * c)
        u1, u2 = u[0::2], u[1::2]
        g = np.sqrt(-2.0 * np.log1p(-u1)) * np.cos(2.0 * np.pi * u2)
        out[s:s + c] = f64_to_bf16_bits(mean + sigma * g)
    return out.reshape(shape)


def small_int_bf16(seed: int, tensor_id: int, shape, lo: int = -2, hi: int = 2) -> np.ndarray:
    """Integers in [lo, hi] (exact in bf16): every partial sum of a product of
    two such tensors is an integer, so fp32 accumulation is exact in any order."""
    n = int(np.prod(shape))
    u = unit_uniform(seed, tensor_id, 0, n)
    v = np.floor(u * (hi - lo + 1)) + lo
    return f64_to_bf16_bits(v).reshape(shape)


@dataclass(frozen=True)
class Workload:
    name: str
    M: int
    N: int
    K: int
    seed: int
    a_dist: tuple   # ("uniform", scale) or ("normal", sigma)
    b_dist: tuple
    bias_dist: tuple
    bound: str      # "mfma", "hbm" or "latency": which roof the shape sits under

    @property
    def flops(self) -> int:
        return 2 * self.M * self.N * self.K

    @property
    def algorithmic_bytes(self) -> int:
        """A, B and bias read once, Y written once, all bf16."""
        return 2 * (self.M * self.K + self.K * self.N + self.M * self.N + self.N)


def _draw(dist, seed, tid, shape):
    kind, p = dist
    if kind == "uniform":
        return uniform_bf16(seed, tid, shape, p)
    if kind == "normal":
        return normal_bf16(seed, tid, shape, p)
    raise ValueError(kind)


WORKLOADS = {
    "C1": Workload("C1", 256, 256, 256, 0, ("uniform", 256 ** -0.5), ("uniform", 256 ** -0.5),
                   ("normal", 1.0), "latency"),
    "C2": Workload("C2", 2048, 2048, 2048, 1, ("uniform", 2048 ** -0.5), ("uniform", 2048 ** -0.5),
                   ("normal", 1.0), "mfma"),
    "C3": Workload("C3", 4096, 11008, 4096, 2, ("normal", 1.0), ("normal", 0.02),
                   ("normal", 0.01), "mfma"),
    "C4": Workload("C4", 16, 8192, 8192, 3, ("normal", 1.0), ("normal", 0.02),
                   ("normal", 0.01), "hbm"),
    "C5": Workload("C5", 1024, 1024, 16384, 4, ("uniform", 16384 ** -0.5), ("uniform", 16384 ** -0.5),
                   ("normal", 1.0), "mfma"),
}


def make_inputs(w: Workload):
    """(A[M,K], B[K,N], bias[N]) as uint16 bf16 bit patterns."""
    A = _draw(w.a_dist, w.seed, 0, (w.M, w.K))
    B = _draw(w.b_dist, w.seed, 1, (w.K, w.N))
    bias = _draw(w.bias_dist, w.seed, 2, (w.N,))
    return A, B, bias


def make_custom(M, N, K, seed, a_dist=("uniform", None), b_dist=("uniform", None),
                bias_dist=("normal", 1.0)):
    """Same recipe as C1 at an arbitrary shape (used for ragged parity cases)."""
    sc = max(K, 1) ** -0.5
    a_dist = ("uniform", sc) if a_dist == ("uniform", None) else a_dist
    b_dist = ("uniform", sc) if b_dist == ("uniform", None) else b_dist
    A = _draw(a_dist, seed, 0, (M, K))
    B = _draw(b_dist, seed, 1, (K, N))
    bias = _draw(bias_dist, seed, 2, (N,))
    return A, B, bias


# ---- batched vector-matrix product (the paper's Case Study 2): C[m, n] = sum_k A[m, k] B[m, n, k].
# The paper gives no shapes; these are chosen here. V1 is small enough for the CPU oracle in well
# under a second and still has several row groups and a ragged last k chunk; V2 reads 1 GiB of B.
@dataclass(frozen=True)
class VecmatWorkload:
    name: str
    M: int
    N: int
    K: int
    seed: int

    @property
    def flops(self) -> int:
        return 2 * self.M * self.N * self.K

    @property
    def algorithmic_bytes(self) -> int:
        """A and B read once (bf16), C written once (fp32)."""
        return 2 * (self.M * self.K + self.M * self.N * self.K) + 4 * self.M * self.N


VECMAT_WORKLOADS = {
    "V1": VecmatWorkload("V1", 8, 520, 1000, 10),
    "V2": VecmatWorkload("V2", 32, 4096, 4096, 11),
}


def make_vecmat(M, N, K, seed):
    """(A[M,K] ~ N(0,1), B[M,N,K] ~ uniform[-1,1)/sqrt(K)) as uint16 bf16 bit patterns."""
    A = normal_bf16(seed, 0, (M, K), 1.0)
    B = uniform_bf16(seed, 1, (M, N, K), max(K, 1) ** -0.5)
    return A, B


# ---- batched product with a transposed first operand (the paper's Case Study 3, dB = dO^T A):
# C[b, m, n] = sum_k A[b, k, m] B[b, k, n], one product per (batch, chunk) item, k = position in the chunk.
# The paper gives no shapes; T1 is the small ragged case, T2 has the flops of the 2048^3 GEMM.
@dataclass(frozen=True)
class BatchedGemmWorkload:
    name: str
    batch: int
    M: int
    N: int
    K: int
    seed: int

    @property
    def flops(self) -> int:
        return 2 * self.batch * self.M * self.N * self.K

    @property
    def algorithmic_bytes(self) -> int:
        """A and B read once (bf16), C written once (fp32)."""
        return self.batch * (2 * self.K * (self.M + self.N) + 4 * self.M * self.N)


BGEMM_WORKLOADS = {
    "T1": BatchedGemmWorkload("T1", 3, 136, 200, 128, 20),
    "T2": BatchedGemmWorkload("T2", 32, 1024, 1024, 256, 21),
}


def make_bgemm(batch, M, N, K, seed):
    """(A[batch,K,M], B[batch,K,N]) ~ N(0,1) resp. uniform[-1,1)/sqrt(K), as uint16 bf16 bit patterns."""
    A = normal_bf16(seed, 0, (batch, K, M), 1.0)
    B = uniform_bf16(seed, 1, (batch, K, N), max(K, 1) ** -0.5)
    return A, B


# ---- element-wise sine (the paper's Case Study 1): y[i] = sin(x[i]), binary32 in and out.
# The paper gives no size; E1 is the small ragged case, E2 moves 512 MB per launch.
@dataclass(frozen=True)
class SinWorkload:
    name: str
    n: int
    seed: int

    @property
    def flops(self) -> int:
        return self.n            # one function evaluation per element

    @property
    def algorithmic_bytes(self) -> int:
        return 8 * self.n        # x read, y written, 4 bytes each


SIN_WORKLOADS = {"E1": SinWorkload("E1", 100003, 30), "E2": SinWorkload("E2", 1 << 26, 31)}


def make_sin_input(n, seed, sigma=10.0):
    """x ~ N(0, sigma) as float32 (same counter-based generator, rounded once from double)."""
    out = np.empty(n, np.float32)
    for s in range(0, n, _CHUNK):
        c = min(_CHUNK, n - s)
        u = unit_uniform(seed, 0, 2 * s, 2 * c)
        u1, u2 = u[0::2], u[1::2]
        out[s:s + c] = (sigma * np.sqrt(-2.0 * np.log1p(-u1)) * np.cos(2.0 * np.pi * u2)).astype(np.float32)
    return out
