// Device-side building blocks of the reduced-precision checkpoint (store type SCAR_F32_BF16C:
// float32 x, bfloat16 c; Example 2.1), shared by the fixed-layout kernels and the walk over
// blocks of unequal length.
#pragma once

#include "scar_device.hpp"

namespace scar {

constexpr int kMixUnit = 4;  // elements per unit: one 16-byte vector of x, 8 bytes of c
constexpr int kMixU = 4;     // units per lane kept in flight by the read-only kernels

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint2 load_stream2(const uint2* p) {
  const u32x2 r = __builtin_nontemporal_load((const u32x2*)p);
  return make_uint2(r.x, r.y);
}
__device__ __forceinline__ void store_stream2(uint2* p, const uint2& v) {
  u32x2 r;
  r.x = v.x, r.y = v.y;
  __builtin_nontemporal_store(r, (u32x2*)p);
}

__device__ __forceinline__ float widen_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float widen_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// float32 bits -> bfloat16 bits, round to nearest even; NaN stays a (quiet) NaN.
__device__ __forceinline__ uint32_t round_bf16(uint32_t u) {
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x0040u;
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// Sum of squared differences of one unit: xv holds 4 floats, cv the matching 4 bfloat16.
__device__ __forceinline__ float sqdiff_unit(const uint4& xv, const uint2& cv) {
  const float d0 = __uint_as_float(xv.x) - widen_lo(cv.x);
  const float d1 = __uint_as_float(xv.y) - widen_hi(cv.x);
  const float d2 = __uint_as_float(xv.z) - widen_lo(cv.y);
  const float d3 = __uint_as_float(xv.w) - widen_hi(cv.y);
  const float s = __builtin_fmaf(d3, d3, __builtin_fmaf(d2, d2, __builtin_fmaf(d1, d1, d0 * d0)));
  return s;
}

__device__ __forceinline__ uint4 widen_unit(const uint2& cv) {
  return make_uint4(cv.x << 16, cv.x & 0xffff0000u, cv.y << 16, cv.y & 0xffff0000u);
}

__device__ __forceinline__ uint2 round_unit(const uint4& xv) {
  return make_uint2(round_bf16(xv.x) | (round_bf16(xv.y) << 16),
                    round_bf16(xv.z) | (round_bf16(xv.w) << 16));
}

__device__ __forceinline__ float widen_elem(const uint16_t* c, uint64_t j) {
  return __uint_as_float((uint32_t)c[j] << 16);
}

}  // namespace scar
