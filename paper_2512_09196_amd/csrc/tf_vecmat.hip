// Batched vector-matrix product (the paper's Case Study 2) for gfx950:
//     C[m][n] = sum_k A[m][k] * B[m][n][k],   A, B bf16, C fp32, fp32 accumulation.
// B is [M][N][ldb] with k contiguous, so the whole cost is reading B once from HBM: 2 flop per
// 2 bytes, far below the ridge; no matrix instruction is involved.
//
//  * naive (the baseline kernel of the variant loop for this operation): one thread per output,
//    a scalar loop over k. Neighbouring threads read rows of B that are ldb elements apart, so
//    every load instruction touches 64 different lines: the uncoalesced starting point.
//  * stream family <R, U, NW>: a wave owns R neighbouring rows (m, n .. n+R-1) at a time and walks
//    k in chunks of 512 elements: lane l loads the 16 bytes at k = 512 c + 8 l of each row (one
//    contiguous KB per row and load) and of A[m] (shared by the R rows), unpacks bf16 to fp32 and
//    accumulates with FMAs; U chunks are in flight per row. The 64 partial sums of a row are added
//    with lane exchanges and lane 0 writes C. A wave takes row groups a grid stride apart, so
//    the grid size is a tunable (one wave per row group, or a grid that just fills the chip).
#include "tf_device.h"

namespace tf {

__global__ void __launch_bounds__(256) tf_vecmat_naive_kernel(const GemmParams p) {
  const int n = blockIdx.x * 256 + threadIdx.x;
  const int m = blockIdx.y;
  if (n >= p.N) return;
  const uint16_t* a = p.A + (size_t)m * p.lda;
  const uint16_t* b = p.B + ((size_t)m * p.N + n) * p.ldb;
  float acc = 0.0f;
  for (int k = 0; k < p.K; ++k) acc = __builtin_fmaf(bf16_bits_to_f32(a[k]), bf16_bits_to_f32(b[k]), acc);
  ((float*)p.Y)[(size_t)m * p.ldy + n] = acc;
}

template <int R_, int U_, int NW_>
struct VecmatCfg {
  static constexpr int R = R_, U = U_, NW = NW_, THREADS = NW_ * 64;
  static_assert(R * U <= 16, "at most 64 registers of B in flight per lane");
};

__device__ __forceinline__ float dot8(const u32x4 a, const u32x4 b, float acc) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    acc = __builtin_fmaf(__builtin_bit_cast(float, a[i] << 16), __builtin_bit_cast(float, b[i] << 16), acc);
    acc = __builtin_fmaf(__builtin_bit_cast(float, a[i] & 0xffff0000u), __builtin_bit_cast(float, b[i] & 0xffff0000u), acc);
  }
  return acc;
}

template <class C>
__global__ void __launch_bounds__(C::THREADS) tf_vecmat_stream_kernel(const GemmParams p) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const long groups_per_m = (p.N + C::R - 1) / C::R;
  const long groups = groups_per_m * p.M;
  const long total_waves = (long)gridDim.x * C::NW;
  const int nchunks = (p.K + 511) / 512;
  for (long g = (long)blockIdx.x * C::NW + wave; g < groups; g += total_waves) {
    const int m = (int)(g / groups_per_m);
    const int n0 = (int)(g % groups_per_m) * C::R;
    const char* arow = (const char*)(p.A + (size_t)m * p.lda) + lane * 16;
    const char* brow[C::R];
#pragma unroll
    for (int r = 0; r < C::R; ++r) {
      int n = n0 + r;
      if (n >= p.N) n = p.N - 1;             // rows past N repeat the last row; nothing is stored for them
      brow[r] = (const char*)(p.B + ((size_t)m * p.N + n) * p.ldb) + lane * 16;
    }
    float acc[C::R];
#pragma unroll
    for (int r = 0; r < C::R; ++r) acc[r] = 0.0f;
    for (int c0 = 0; c0 < nchunks; c0 += C::U) {
      u32x4 av[C::U], bv[C::R][C::U];
#pragma unroll
      for (int u = 0; u < C::U; ++u) {
        const int k = (c0 + u) * 512 + lane * 8;       // K is a multiple of 8: 16 bytes are all in or all out
        const bool in = k < p.K;
        const size_t off = (size_t)(c0 + u) * 1024;
        av[u] = in ? *(const u32x4*)(arow + off) : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int r = 0; r < C::R; ++r) bv[r][u] = in ? __builtin_nontemporal_load((const u32x4*)(brow[r] + off)) : u32x4{0u, 0u, 0u, 0u};
      }
#pragma unroll
      for (int u = 0; u < C::U; ++u)
#pragma unroll
        for (int r = 0; r < C::R; ++r) acc[r] = dot8(av[u], bv[r][u], acc[r]);
    }
#pragma unroll
    for (int r = 0; r < C::R; ++r) {
      float s = acc[r];
#pragma unroll
      for (int d = 32; d >= 1; d >>= 1) s += __shfl_xor(s, d, 64);
      if (lane == 0 && n0 + r < p.N) ((float*)p.Y)[(size_t)m * p.ldy + n0 + r] = s;
    }
  }
}

template <class C>
static void launch_vecmat(const GemmParams& p, dim3 grid, hipStream_t stream) {
  hipLaunchKernelGGL(tf_vecmat_stream_kernel<C>, grid, dim3(C::THREADS), 0, stream, p);
}

template <class C>
static VecmatKernelInfo make_vecmat_info() {
  VecmatKernelInfo k;
  k.rows = C::R; k.unroll = C::U; k.waves = C::NW; k.threads = C::THREADS;
  k.func = (const void*)tf_vecmat_stream_kernel<C>;
  k.launch = launch_vecmat<C>;
  return k;
}

static VecmatKernelInfo g_vecmat_table[] = {
    make_vecmat_info<VecmatCfg<1, 2, 4>>(), make_vecmat_info<VecmatCfg<1, 4, 4>>(),
    make_vecmat_info<VecmatCfg<1, 8, 4>>(), make_vecmat_info<VecmatCfg<2, 4, 4>>(),
    make_vecmat_info<VecmatCfg<2, 8, 4>>(), make_vecmat_info<VecmatCfg<4, 4, 4>>(),
    make_vecmat_info<VecmatCfg<4, 2, 8>>(), make_vecmat_info<VecmatCfg<2, 4, 8>>(),
    make_vecmat_info<VecmatCfg<1, 8, 8>>(),
};

int vecmat_kernel_count() { return (int)(sizeof(g_vecmat_table) / sizeof(g_vecmat_table[0])); }
const VecmatKernelInfo* vecmat_kernel_table() { return g_vecmat_table; }
void launch_vecmat_naive(const GemmParams& p, hipStream_t s) {
  hipLaunchKernelGGL(tf_vecmat_naive_kernel, dim3((unsigned)((p.N + 255) / 256), (unsigned)p.M), dim3(256), 0, s, p);
}
const void* vecmat_naive_func() { return (const void*)tf_vecmat_naive_kernel; }

}  // namespace tf
