// Device-side helpers common to all kernels of the family (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "tf_internal.h"

namespace tf {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) {
  return __builtin_bit_cast(float, (uint32_t)b << 16);
}

// fp32 -> bf16, round to nearest even; NaN stays a quiet NaN.
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  uint32_t w = __builtin_bit_cast(uint32_t, f);
  if ((w & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((w >> 16) | 0x0040u);
  w += 0x7fffu + ((w >> 16) & 1u);
  return (uint16_t)(w >> 16);
}

// Two fp32 -> packed bf16 (round to nearest even, NaN kept quiet): one v_cvt_pk_bf16_f32.
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
}

// GELU(z) = z * Phi(z) with the exact-erf definition, Phi(z) = erfc(-z / sqrt 2) / 2.
// Written as  GELU(z) = max(z, 0) - |z| * Phi(-|z|)  (both signs of z give this), so the
// negative tail keeps its relative accuracy and no select is needed.
// Phi(-u), u >= 0, is evaluated as exp2(-p(u)): -log2 Phi(-u) is smooth and grows like u^2, so
// a degree-7 polynomial p (minimax fit on [0, 5.5] against the double-precision log of the
// normal CDF, |error| < 5e-6, i.e. 3.3e-6 relative in Phi) and ONE transcendental instruction
// do it; a transcendental costs four issue slots of a 64-lane wave, the seven FMAs one each.
// Past u = 5.5 the term is frozen at 5.5 * Phi(-5.5) = 1.0e-7, which is also a bound on the
// true value there. Measured against the double-precision definition over [-40, 40]:
// |error| <= 3.8e-7 (1 + |z|), relative error <= 6.4e-6 on the negative side.
// max(z, 0) is taken as (z + |z|) / 2, which is exact and, unlike v_max_f32, keeps a NaN.
__device__ __forceinline__ float gelu_erf(float z) {
  const float u = __builtin_fabsf(z);
  const float uc = __builtin_fminf(u, 5.5f);
  float p = -1.793487627e-06f;
  p = __builtin_fmaf(p, uc, 6.090477109e-05f);
  p = __builtin_fmaf(p, uc, -9.260333027e-04f);
  p = __builtin_fmaf(p, uc, 8.493772708e-03f);
  p = __builtin_fmaf(p, uc, -5.393787101e-02f);
  p = __builtin_fmaf(p, uc, -4.584804773e-01f);
  p = __builtin_fmaf(p, uc, -1.151246786e+00f);
  p = __builtin_fmaf(p, uc, -9.999954700e-01f);     // log2 Phi(-uc)
  const float tail = uc * __builtin_amdgcn_exp2f(p);   // |z| Phi(-|z|)
  return __builtin_fmaf(0.5f, z + u, -tail);
}

// The tanh form of GELU, z/2 (1 + tanh u) with u = sqrt(2/pi) (z + 0.044715 z^3), written as
// z * sigmoid(2u) = z / (1 + 2^(-2u log2 e)): one exp2 and one reciprocal. z is clamped below for the
// product only, so that -inf gives -0 rather than inf * 0 (the true value is below 1e-38 long before);
// a NaN propagates through u. |error| <= 4e-7 |z| against the double-precision definition.
__device__ __forceinline__ float gelu_tanh(float z) {
  const float u = 0.7978845608f * __builtin_fmaf(0.044715f * z * z, z, z);
  const float e = __builtin_amdgcn_exp2f(-2.885390082f * u);
  return __builtin_fmaxf(z, -1.0e4f) * __builtin_amdgcn_rcpf(1.0f + e);
}

// The activation of a bf16 epilogue, chosen at compile time (tile kernels) or at run time (the small kernels).
template <int EPI>
__device__ __forceinline__ float activate(float z) {
  if (EPI == TF_EPI_BIAS_GELU_ERF) return gelu_erf(z);
  if (EPI == TF_EPI_BIAS_GELU_TANH) return gelu_tanh(z);
  return z;
}
__device__ __forceinline__ float activate(float z, int epi) {
  if (epi == TF_EPI_BIAS_GELU_ERF) return gelu_erf(z);
  if (epi == TF_EPI_BIAS_GELU_TANH) return gelu_tanh(z);
  return z;
}

// Work-group id -> position in the tile order.
//  * The hardware deals consecutive work-group ids round-robin over the 8 XCDs, each with
//    its own L2. With xcd_swizzle the ids are renumbered so that each XCD owns one
//    contiguous run of the tile order, and tiles that share an A row panel or a B column
//    panel hit the same L2.
//  * Within the order, tiles advance down a column of `group_m` tile rows before moving to
//    the next tile column, so a group re-uses its A panels while B panels stream.
struct TileCoord { int tm, tn, ks; };

// Position t in the grouped tile order -> tile coordinates (ks = 0).
__device__ __forceinline__ TileCoord tile_at(const GemmParams& p, int t) {
  TileCoord c;
  c.ks = 0;
  const int gsz = p.group_m * p.tiles_n;
  const int g = t / gsz;
  const int first_m = g * p.group_m;
  const int rows = (p.tiles_m - first_m) < p.group_m ? (p.tiles_m - first_m) : p.group_m;
  const int in_g = t - g * gsz;
  c.tm = first_m + in_g % rows;
  c.tn = in_g / rows;
  return c;
}
// id in [0, total) -> the same range renumbered so that XCD (id mod 8) owns one contiguous run
__device__ __forceinline__ int xcd_run(int id, int total) {
  const int xcd = id & 7, local = id >> 3;
  const int base = total >> 3, rem = total & 7;
  return xcd * base + (xcd < rem ? xcd : rem) + local;
}

__device__ __forceinline__ TileCoord map_tile(const GemmParams& p, int wg) {
  const int tiles = p.tiles_m * p.tiles_n;
  const int total = tiles * p.split_k;
  int id = wg;
  if (p.xcd_swizzle) {
    const int nx = 8;
    const int xcd = wg % nx, local = wg / nx;
    const int base = total / nx, rem = total % nx;
    // XCD x owns base + (x < rem) consecutive ids
    id = xcd * base + (xcd < rem ? xcd : rem) + local;
  }
  TileCoord c;
  int t;
  if (p.slice_major) {
    // all tiles of K slice 0, then all of slice 1, ...: work-groups that share an XCD's L2 work on the same K range
    // of neighbouring tiles and re-use each other's A and B panels (the slices of a tile need not meet: a second
    // kernel sums them)
    c.ks = id / tiles;
    t = id - c.ks * tiles;
  } else {
    c.ks = id % p.split_k;        // slices of one tile are neighbours: they finish together
    t = id / p.split_k;
  }
  const int gsz = p.group_m * p.tiles_n;
  const int g = t / gsz;
  const int first_m = g * p.group_m;
  const int rows = (p.tiles_m - first_m) < p.group_m ? (p.tiles_m - first_m) : p.group_m;
  const int in_g = t - g * gsz;
  c.tm = first_m + in_g % rows;
  c.tn = in_g / rows;
  return c;
}

}  // namespace tf
