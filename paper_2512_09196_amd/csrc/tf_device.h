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
// erfc(x), x >= 0, by the rational-exponential form of Abramowitz & Stegun 7.1.26:
//   erfc(x) = (a1 t + a2 t^2 + a3 t^3 + a4 t^4 + a5 t^5) exp(-x^2),  t = 1 / (1 + p x),
// absolute error below 1.5e-7 for every x >= 0. With x = |z| / sqrt 2:
//   |z| * Phi(-|z|) = x * (sqrt 2 / 2) * erfc(x);  the factor sqrt(2)/2 is folded into a1..a5.
__device__ __forceinline__ float gelu_erf(float z) {
  const float x = __builtin_fabsf(z) * 0.70710678118654752f;
  const float t = __builtin_amdgcn_rcpf(__builtin_fmaf(0.3275911f, x, 1.0f));
  float poly = 0.750526976f;                       // a5 / sqrt 2
  poly = __builtin_fmaf(poly, t, -1.027533652f);   // a4 / sqrt 2
  poly = __builtin_fmaf(poly, t, 1.005091295f);    // a3 / sqrt 2
  poly = __builtin_fmaf(poly, t, -0.201169571f);   // a2 / sqrt 2
  poly = __builtin_fmaf(poly, t, 0.180191733f);    // a1 / sqrt 2
  // exp(-x^2) = exp2(-x^2 log2 e); arguments below -126 flush to zero, which is the limit
  const float e = __builtin_amdgcn_exp2f(-1.44269504088896341f * x * x);
  const float tail = poly * t * e * x;             // |z| Phi(-|z|)
  return __builtin_fmaxf(z, 0.0f) - tail;
}

// Work-group id -> position in the tile order.
//  * The hardware deals consecutive work-group ids round-robin over the 8 XCDs, each with
//    its own L2. With xcd_swizzle the ids are renumbered so that each XCD owns one
//    contiguous run of the tile order, and tiles that share an A row panel or a B column
//    panel hit the same L2.
//  * Within the order, tiles advance down a column of `group_m` tile rows before moving to
//    the next tile column, so a group re-uses its A panels while B panels stream.
struct TileCoord { int tm, tn, ks; };

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
  c.ks = id % p.split_k;          // slices of one tile are neighbours: they finish together
  const int t = id / p.split_k;
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
