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

// Elements of a row before its first whole unit (4 elements: 16 bytes of x on a 16-byte
// boundary, 8 bytes of c on an 8-byte boundary).  Both streams reach such boundaries at the same
// elements exactly when the two row addresses have the same phase, counted in elements modulo
// 4; then the row is walked in units between (-phase) mod 4 leading and a few trailing
// elements, whatever its length.  Rows whose phases differ (views that start at unrelated
// offsets, packed rows of a length that is no multiple of 4) are walked element by element: all
// of the row is "head".  Decided per row from the addresses, so every kernel splits a given row
// in the same way.
__device__ __forceinline__ uint32_t mixed_head(const float* xb, const uint16_t* cb, uint32_t len) {
  const uint32_t px = (uint32_t)((uintptr_t)xb >> 2) & (kMixUnit - 1);
  const uint32_t pc = (uint32_t)((uintptr_t)cb >> 1) & (kMixUnit - 1);
  if (px != pc) return len;
  const uint32_t head = (0u - px) & (kMixUnit - 1);
  return head < len ? head : len;
}

// Squared distance of one block (len elements at xb / cb, the first `head` of them before the
// first whole unit), this lane's share: the whole units, then the elements around them.
template <int G>
__device__ __forceinline__ double mixed_distance(const float* xb, const uint16_t* cb, uint32_t len,
                                                 uint32_t head, int lane) {
  double acc = 0;
  const uint32_t nunit = (len - head) / kMixUnit;
  const uint32_t tail0 = head + nunit * kMixUnit;
  const uint4* xv = (const uint4*)(xb + head);
  const uint2* cv = (const uint2*)(cb + head);
  for (uint32_t u0 = 0; u0 < nunit; u0 += G * kMixU) {
    uint4 a[kMixU];
    uint2 b[kMixU];
#pragma unroll
    for (int u = 0; u < kMixU; ++u) {
      const uint32_t i = u0 + u * G + lane;
      if (i < nunit) {
        a[u] = load_stream(xv + i);
        b[u] = load_stream2(cv + i);
      } else {
        a[u] = make_uint4(0, 0, 0, 0);
        b[u] = make_uint2(0, 0);
      }
    }
    float part = 0.f;
#pragma unroll
    for (int u = 0; u < kMixU; ++u) part += sqdiff_unit(a[u], b[u]);
    acc += (double)part;
  }
  for (uint32_t e = lane; e < len - nunit * kMixUnit; e += G) {
    const uint32_t j = e < head ? e : tail0 + (e - head);
    acc += (double)sq(xb[j] - widen_elem(cb, j));
  }
  return acc;
}

}  // namespace scar
