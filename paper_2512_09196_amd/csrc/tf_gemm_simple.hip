// The two unstaged members of the family.
//
//  * naive: the baseline kernel K of the variant loop. One thread per output element, a
//    scalar fp32 FMA loop over K, no MFMA, no LDS; accepts any shape, stride and alignment.
//  * mfma_direct: one wave per 32x32 output tile; MFMA operands are gathered straight from
//    memory, element by element, with guards, so it also accepts any shape. It exists to pin
//    the MFMA operand and accumulator lane layouts with nothing else in the way.
#include "tf_device.h"

namespace tf {

__global__ void __launch_bounds__(256) tf_gemm_naive_kernel(const GemmParams p) {
  const int n = blockIdx.x * 64 + (threadIdx.x & 63);
  const int m = blockIdx.y * 4 + (threadIdx.x >> 6);
  if (m >= p.M || n >= p.N) return;
  const uint16_t* a = p.A + (size_t)m * p.lda;
  const uint16_t* b = p.B + n;
  float acc = 0.0f;
  for (int k = 0; k < p.K; ++k)
    acc = __builtin_fmaf(bf16_bits_to_f32(a[k]), bf16_bits_to_f32(b[(size_t)k * p.ldb]), acc);
  const float z = acc + bf16_bits_to_f32(p.bias[n]);
  if (p.epi == TF_EPI_NONE_F32) ((float*)p.Y)[(size_t)m * p.ldy + n] = z;
  else ((uint16_t*)p.Y)[(size_t)m * p.ldy + n] = f32_to_bf16_bits(gelu_erf(z));
}

__global__ void __launch_bounds__(64) tf_gemm_mfma_direct_kernel(const GemmParams p) {
  const int lane = threadIdx.x;
  const int m0 = blockIdx.y * 32, n0 = blockIdx.x * 32;
  const int r = lane & 31, g = lane >> 5;
  // v_mfma_f32_32x32x16_bf16 operand layout: lane l supplies row (A) / column (B) l % 32
  // and the eight k values 8 (l / 32) .. 8 (l / 32) + 7 of the 16-wide k step.
  const int am = m0 + r, bn = n0 + r;
  f32x16 acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.0f;
  for (int k0 = 0; k0 < p.K; k0 += 16) {
    s16x8 av, bv;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int k = k0 + 8 * g + e;
      const bool kin = k < p.K;
      av[e] = (kin && am < p.M) ? (short)p.A[(size_t)am * p.lda + k] : (short)0;
      bv[e] = (kin && bn < p.N) ? (short)p.B[(size_t)k * p.ldb + bn] : (short)0;
    }
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), __builtin_bit_cast(bf16x8, bv), acc, 0, 0, 0);
  }
  // accumulator layout: register i of lane l is row 8 (i / 4) + 4 (l / 32) + i % 4, column l % 32
  const int n = n0 + r;
  if (n >= p.N) return;
  const float bias = bf16_bits_to_f32(p.bias[n]);
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int m = m0 + 8 * (i >> 2) + 4 * g + (i & 3);
    if (m < p.M) {
      const float z = acc[i] + bias;
      if (p.epi == TF_EPI_NONE_F32) ((float*)p.Y)[(size_t)m * p.ldy + n] = z;
      else ((uint16_t*)p.Y)[(size_t)m * p.ldy + n] = f32_to_bf16_bits(gelu_erf(z));
    }
  }
}

__global__ void tf_fill_u32_kernel(unsigned* p, size_t n, unsigned v) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

void launch_naive(const GemmParams& p, hipStream_t s) {
  dim3 grid((p.N + 63) / 64, (p.M + 3) / 4);
  hipLaunchKernelGGL(tf_gemm_naive_kernel, grid, dim3(256), 0, s, p);
}
void launch_mfma_direct(const GemmParams& p, hipStream_t s) {
  dim3 grid((p.N + 31) / 32, (p.M + 31) / 32);
  hipLaunchKernelGGL(tf_gemm_mfma_direct_kernel, grid, dim3(64), 0, s, p);
}
const void* naive_func() { return (const void*)tf_gemm_naive_kernel; }
const void* mfma_direct_func() { return (const void*)tf_gemm_mfma_direct_kernel; }
void launch_fill_u32(unsigned* p, size_t n, unsigned v, hipStream_t s) {
  if (n == 0) return;
  hipLaunchKernelGGL(tf_fill_u32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p, n, v);
}

}  // namespace tf
