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

// Second kernel of the two-kernel split-K: Y = epilogue(sum_s ws[s] + bias), slices summed in
// slice order. One thread per four consecutive n (N is a multiple of 8 for every tile kernel).
__global__ void __launch_bounds__(256) tf_splitk_reduce_kernel(const GemmParams p) {
  const size_t quads_per_row = (size_t)p.N / 4;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)p.M * quads_per_row) return;
  const size_t m = i / quads_per_row;
  const int n = (int)(i % quads_per_row) * 4;
  const size_t slice = (size_t)p.M * p.N;
  const float* src = p.ws + m * p.N + n;
  f32x4 sum = {0.0f, 0.0f, 0.0f, 0.0f};
  for (int s = 0; s < p.split_k; ++s) sum += *(const f32x4*)(src + (size_t)s * slice);
  const u32x2 braw = *(const u32x2*)(p.bias + n);
  const float z0 = sum[0] + __builtin_bit_cast(float, braw[0] << 16);
  const float z1 = sum[1] + __builtin_bit_cast(float, braw[0] & 0xffff0000u);
  const float z2 = sum[2] + __builtin_bit_cast(float, braw[1] << 16);
  const float z3 = sum[3] + __builtin_bit_cast(float, braw[1] & 0xffff0000u);
  if (p.epi == TF_EPI_NONE_F32) {
    const f32x4 v = {z0, z1, z2, z3};
    *(f32x4*)((float*)p.Y + m * p.ldy + n) = v;
  } else {
    u32x2 o;
    o[0] = pack_bf16x2(gelu_erf(z0), gelu_erf(z1));
    o[1] = pack_bf16x2(gelu_erf(z2), gelu_erf(z3));
    *(u32x2*)((uint16_t*)p.Y + m * p.ldy + n) = o;
  }
}

void launch_splitk_reduce(const GemmParams& p, hipStream_t s) {
  const size_t quads = (size_t)p.M * (p.N / 4);
  hipLaunchKernelGGL(tf_splitk_reduce_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, s, p);
}
const void* splitk_reduce_func() { return (const void*)tf_splitk_reduce_kernel; }

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
