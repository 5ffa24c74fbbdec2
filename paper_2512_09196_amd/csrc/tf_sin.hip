// Element-wise sine (the paper's Case Study 1) for gfx950: y[i] = sin(x[i]), binary32 in and out.
// The arithmetic is the same in every kernel; what varies is the launch shape, which is the whole
// point of the case: its baseline gives every work-group four elements.
//
// sin x: q = nearest integer to x * 2/pi; r = x - q * pi/2 by three FMAs against a three-part
// pi/2 (each step rounds once; good to |x| of about 1e4); then a degree-7 odd polynomial for
// sin r or a degree-8 even one for cos r on |r| <= pi/4, chosen by q mod 2, sign by q mod 4.
// Coefficients: minimax fits of (sin r / r - 1) / r^2 and (cos r - 1 + r^2/2) / r^4 in r^2.
// Measured against the double-precision sine over N(0, 1000) inputs: |error| <= 9.3e-8.
#include "tf_device.h"

namespace tf {

__device__ __forceinline__ float sin_f32(float x) {
  const float q = __builtin_rintf(x * 0.6366197723675814f);
  float r = __builtin_fmaf(-q, 1.5707963705062866f, x);
  r = __builtin_fmaf(-q, -4.371138828673793e-08f, r);
  r = __builtin_fmaf(-q, -1.7763568394002505e-15f, r);
  const float u = r * r;
  float s = __builtin_fmaf(u, -0.00019582954701036215f, 0.008332725614309311f);
  s = __builtin_fmaf(s, u, -0.166666641831398f);
  const float sv = __builtin_fmaf(s * u, r, r);
  float c = __builtin_fmaf(u, 2.456760012137238e-05f, -0.0013888463145121932f);
  c = __builtin_fmaf(c, u, 0.0416666679084301f);
  const float cv = __builtin_fmaf(c * u, u, __builtin_fmaf(u, -0.5f, 1.0f));
  const int n = (int)q;
  const float y = x == 0.0f ? x : ((n & 1) ? cv : sv);     // the reduction turns -0 into +0: keep the sign of a zero argument
  return __builtin_bit_cast(float, __builtin_bit_cast(unsigned, y) ^ ((unsigned)(n & 2) << 30));
}

// The baseline: BLOCK_SIZE = 4. One 64-lane wave per work-group, four lanes busy.
__global__ void __launch_bounds__(64) tf_sin_block4_kernel(const float* x, float* y, size_t n) {
  const size_t i = (size_t)blockIdx.x * 4 + threadIdx.x;
  if (threadIdx.x < 4 && i < n) y[i] = sin_f32(x[i]);
}

// THREADS threads, VEC consecutive elements per thread and pass, ITERS passes per work-group
// (BLOCK_SIZE = THREADS * VEC * ITERS), then a grid stride to the work-group's next block. NT marks the
// accesses non-temporal: every element is touched once, so nothing is worth keeping in the caches.
template <int THREADS, int VEC, int ITERS, bool NT>
__global__ void __launch_bounds__(THREADS) tf_sin_kernel(const float* x, float* y, size_t n) {
  typedef float vec __attribute__((ext_vector_type(VEC)));
  constexpr size_t BLOCK = (size_t)THREADS * VEC * ITERS;
  for (size_t base = (size_t)blockIdx.x * BLOCK; base < n; base += (size_t)gridDim.x * BLOCK) {
    vec v[ITERS];
    bool whole[ITERS];
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
      const size_t i = base + ((size_t)it * THREADS + threadIdx.x) * VEC;
      whole[it] = i + VEC <= n;
      if (whole[it]) {
        if constexpr (NT) v[it] = __builtin_nontemporal_load((const vec*)(x + i));
        else v[it] = *(const vec*)(x + i);
      }
    }
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
      const size_t i = base + ((size_t)it * THREADS + threadIdx.x) * VEC;
      if (whole[it]) {
        vec o;
#pragma unroll
        for (int e = 0; e < VEC; ++e) o[e] = sin_f32(v[it][e]);
        if constexpr (NT) __builtin_nontemporal_store(o, (vec*)(y + i));
        else *(vec*)(y + i) = o;
      } else {
        for (int e = 0; e < VEC; ++e)
          if (i + e < n) y[i + e] = sin_f32(x[i + e]);     // ragged end
      }
    }
  }
}

template <int THREADS, int VEC, int ITERS, bool NT>
static void launch_sin(const float* x, float* y, size_t n, unsigned grid, hipStream_t s) {
  hipLaunchKernelGGL((tf_sin_kernel<THREADS, VEC, ITERS, NT>), dim3(grid), dim3(THREADS), 0, s, x, y, n);
}

template <int THREADS, int VEC, int ITERS, bool NT = false>
static SinKernelInfo make_sin_info() {
  SinKernelInfo k;
  k.threads = THREADS; k.vec = VEC; k.iters = ITERS; k.block = THREADS * VEC * ITERS; k.nontemporal = NT ? 1 : 0;
  k.func = (const void*)tf_sin_kernel<THREADS, VEC, ITERS, NT>;
  k.launch = launch_sin<THREADS, VEC, ITERS, NT>;
  return k;
}

static SinKernelInfo g_sin_table[] = {
    make_sin_info<64, 1, 1>(),    make_sin_info<256, 1, 1>(),  make_sin_info<256, 2, 1>(),  make_sin_info<256, 4, 1>(),
    make_sin_info<256, 4, 4>(),   make_sin_info<512, 4, 2>(),  make_sin_info<1024, 4, 1>(), make_sin_info<1024, 4, 4>(),
    make_sin_info<256, 4, 8>(),   make_sin_info<256, 4, 1, true>(), make_sin_info<256, 4, 2, true>(), make_sin_info<1024, 4, 1, true>(),
    make_sin_info<256, 4, 2>(),
};

int sin_kernel_count() { return (int)(sizeof(g_sin_table) / sizeof(g_sin_table[0])); }
const SinKernelInfo* sin_kernel_table() { return g_sin_table; }
void launch_sin_block4(const float* x, float* y, size_t n, hipStream_t s) {
  hipLaunchKernelGGL(tf_sin_block4_kernel, dim3((unsigned)((n + 3) / 4)), dim3(64), 0, s, x, y, n);
}
const void* sin_block4_func() { return (const void*)tf_sin_block4_kernel; }

}  // namespace tf
