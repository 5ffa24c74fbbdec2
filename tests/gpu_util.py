"""Shared helpers of the GPU parity tests: device buffers, tolerances, canaries."""
import numpy as np

from paper_2512_09196_amd import tf
from paper_2512_09196_amd import workloads as wl

CANARY_BF16 = 0x7FC1      # a NaN pattern no kernel writes
CANARY_F32 = np.float32(-1.2345678e30)


def torch_mod():
    import torch
    return torch


def to_dev(bits: np.ndarray):
    """uint16 bit patterns -> int16 CUDA tensor holding the same bits."""
    torch = torch_mod()
    return torch.from_numpy(bits.view(np.int16).copy()).cuda()


def strided(bits: np.ndarray, ld: int, fill=0x7FC1):
    """Copy a 2-D uint16 array into rows of length ld; the padding holds NaN patterns, so a
    kernel that reads across a row end poisons its result."""
    out = np.full((bits.shape[0], ld), fill, np.uint16)
    out[:, :bits.shape[1]] = bits
    return out


class OutBuf:
    """Y with guard rows before and after and (optionally) padding columns, all canaries."""

    def __init__(self, M, N, ldy=None, f32=False, guard=4):
        torch = torch_mod()
        self.M, self.N, self.ldy, self.f32, self.guard = M, N, N if ldy is None else ldy, f32, guard
        rows = M + 2 * guard
        if f32:
            self.t = torch.full((rows, self.ldy), float(CANARY_F32), dtype=torch.float32, device="cuda")
        else:
            self.t = torch.full((rows, self.ldy), CANARY_BF16,
                                dtype=torch.int16, device="cuda")
        self.ptr = self.t.data_ptr() + guard * self.ldy * (4 if f32 else 2)

    def reset(self):
        if self.f32:
            self.t.fill_(float(CANARY_F32))
        else:
            self.t.fill_(CANARY_BF16)

    def host(self):
        """(values float64 [M,N], guards_intact: bool, raw bits/values [M,N])"""
        torch_mod().cuda.synchronize()
        a = self.t.cpu().numpy()
        g = self.guard
        body = a[g:g + self.M]
        if self.f32:
            intact = bool(np.all(a[:g] == CANARY_F32) and np.all(a[g + self.M:] == CANARY_F32)
                          and np.all(body[:, self.N:] == CANARY_F32))
            raw = body[:, :self.N].copy()
            return raw.astype(np.float64), intact, raw
        u = a.view(np.uint16)
        ub = u[g:g + self.M]
        intact = bool(np.all(u[:g] == CANARY_BF16) and np.all(u[g + self.M:] == CANARY_BF16)
                      and np.all(ub[:, self.N:] == CANARY_BF16))
        raw = ub[:, :self.N].copy()
        return wl.bf16_bits_to_f32(raw).astype(np.float64), intact, raw


def oracle_parallel(A, B, bias, threads=None, block=16, trans_b=False):
    """The unchanged oracle on disjoint row blocks from several host threads (rows are independent; the C function
    holds no state and ctypes releases the interpreter lock). Returns (y, z, s) float64 [M, N] like the oracle."""
    import os
    from concurrent.futures import ThreadPoolExecutor
    from oracle import gemm_oracle as orc
    fn = orc.gemm_nt_bias_gelu if trans_b else orc.gemm_bias_gelu
    M = A.shape[0]
    N = B.shape[0] if trans_b else B.shape[1]
    threads = threads or max(1, min(16, os.cpu_count() or 1))
    y = np.empty((M, N), np.float64)
    z = np.empty((M, N), np.float64)
    s = np.empty((M, N), np.float64)

    def work(r0):
        r1 = min(M, r0 + block)
        yy, zz, ss = fn(A[r0:r1], B, bias)
        y[r0:r1], z[r0:r1], s[r0:r1] = yy, zz, ss
    with ThreadPoolExecutor(max_workers=threads) as ex:
        list(ex.map(work, range(0, M, block)))
    return y, z, s


def gamma(n):
    u = 2.0 ** -24
    return n * u / (1.0 - n * u)


def official_ok(got, y):
    """max |gpu - oracle| <= 1e-2 (1 + |oracle|), elementwise."""
    return np.all(np.abs(got - y) <= 1e-2 * (1.0 + np.abs(y)))


def strict_bound(y, z, s, K):
    """A-priori bound for a correct fp32-accumulating kernel with bf16 output:
    bf16 rounding (half an ulp, 2^-9 relative; 2^-8 taken) + any-order fp32 summation
    (gamma_{K+1} s, doubled: the matrix instruction adds sixteen products to the accumulator in an
    order and with an intermediate rounding that are not documented, so each of its additions is
    allowed a whole unit in the last place instead of half of one) through GELU (slope <= 1.13) +
    the kernel's own evaluation of the activation in fp32 (a polynomial for log2 Phi and one exp2,
    within 3.8e-7 (1 + |z|) of the definition; 1e-6 (1 + |z|) taken)."""
    return 2.0 ** -8 * np.abs(y) + 1.13 * 2.0 * gamma(K + 1) * s + 1e-6 * (1.0 + np.abs(z))


def preact_bound(z, s, K):
    return 2.0 * gamma(K + 1) * s + 2.0 ** -23 * np.abs(z) + 1e-30


def run_variant(prob, vid, dA, dB, dbias, out: OutBuf, **kw):
    out.reset()
    prob.run(vid, dA, dB, dbias, out.ptr, **kw)
    return out.host()
