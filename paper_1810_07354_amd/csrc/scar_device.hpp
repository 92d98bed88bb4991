// Device-side building blocks shared by the SCAR kernels (gfx950, wave64).
//
// A *group* is G consecutive lanes (G = 1..64 inside one wavefront, or G = 256 = the
// whole workgroup) that together walk one block of x and c.  Group sizes are chosen on
// the host so that every lane issues about four 16-byte loads per stream.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace scar {

constexpr int kWG = 256;    // threads per workgroup, 4 wavefronts
constexpr int kWave = 64;
constexpr int kUnroll = 4;  // 16-byte loads per lane and stream kept in flight

// What a kernel measures: squared L2 on float32 / bfloat16, exact L1 on int32 counts, or
// (the *_TV kinds) the total variation 1/2 * sum |x - c| of float rows that are distributions.
// DT_MIXED (only in the walk over blocks of unequal length): float32 x against a bfloat16 c.
enum : int { DT_F32 = 0, DT_BF16 = 1, DT_I32 = 2, DT_F32_TV = 3, DT_BF16_TV = 4, DT_MIXED = 5 };

// Element size of x, and of c (they differ for DT_MIXED only).
__host__ __device__ constexpr int elem_bytes(int dt) { return (dt == DT_BF16 || dt == DT_BF16_TV) ? 2 : 4; }
__host__ __device__ constexpr int c_elem_bytes(int dt) { return dt == DT_MIXED ? 2 : elem_bytes(dt); }
__host__ __device__ constexpr bool is_tv(int dt) { return dt == DT_F32_TV || dt == DT_BF16_TV; }

// ---- streaming memory access ---------------------------------------------------------
// Every byte of x and c is touched once per kernel, so all 16-byte accesses carry the
// non-temporal hint: on MI355X that alone lifts a two-stream read from ~6.3 to ~6.7 TB/s.

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint4 load_stream(const uint4* p) {
  const u32x4 r = __builtin_nontemporal_load((const u32x4*)p);
  return make_uint4(r.x, r.y, r.z, r.w);
}

__device__ __forceinline__ void store_stream(uint4* p, const uint4& v) {
  u32x4 r;
  r.x = v.x, r.y = v.y, r.z = v.z, r.w = v.w;
  __builtin_nontemporal_store(r, (u32x4*)p);
}

// Workgroups are handed to the 8 XCDs round-robin by blockIdx.x.  This renumbering gives
// each XCD one contiguous eighth of the work, so every XCD (own L2, own TLB) streams
// through its own address range instead of all eight striding over the whole store
// (another ~5% on the two-stream read).  gridDim.x must be a multiple of 8.
constexpr uint32_t kXcds = 8;
__device__ __forceinline__ uint32_t xcd_contiguous_block_id() {
  return (blockIdx.x % kXcds) * (gridDim.x / kXcds) + blockIdx.x / kXcds;
}

// The two-dimensional grids of the row kernels: x runs over the index list (`need_x` slots
// hold entries, the rest is padding up to a multiple of 8), y over the pieces of a long row.
// The hardware hands workgroups to the XCDs in the order x fastest, so with x renumbered as
// above an XCD owns an eighth of the list with all its pieces - right for long lists.  A
// short list of very long rows (two lost shards of 256 MiB) would leave the work to the XCDs
// that own x = 0 and x = 1; there the host does not pad x, makes gridDim.y a multiple of 8, and
// the whole grid is renumbered so that each XCD walks a contiguous eighth of the pieces of
// every row.
struct GridSlot {
  uint32_t x, y;
};
__device__ __forceinline__ GridSlot row_grid_slot(uint64_t need_x) {
  if (gridDim.y == 1 || need_x >= 256) return {xcd_contiguous_block_id(), blockIdx.y};  // host: row_grid
  const uint32_t total = gridDim.x * gridDim.y;
  const uint32_t lin = blockIdx.y * gridDim.x + blockIdx.x;
  const uint32_t id = (lin % kXcds) * (total / kXcds) + lin / kXcds;
  return {id % gridDim.x, id / gridDim.x};
}

// ---- per-element distance terms --------------------------------------------------

// The square is rounded to float32 on its own, never fused into a following addition: where
// the compiler can see two of these added up (a lane holding a whole short row) it would
// otherwise make one a fused multiply-add, and the same row scored by a kernel that walks it
// in a loop would round differently (seen on 8-byte float32 rows: one ulp in 8 % of them).
__device__ __forceinline__ float sq(float d) {
#pragma clang fp contract(off)
  return d * d;
}

// Sums of squares are written with explicit fused multiply-adds, so that every kernel that
// measures a block rounds in the same places whatever else it does with the data (the norm
// alone and the norm fused into the recovery agree bit for bit).

// Four float32 lanes of a 16-byte vector.
__device__ __forceinline__ float sqdiff_f32(const uint4& a, const uint4& b) {
  const float d0 = __uint_as_float(a.x) - __uint_as_float(b.x);
  const float d1 = __uint_as_float(a.y) - __uint_as_float(b.y);
  const float d2 = __uint_as_float(a.z) - __uint_as_float(b.z);
  const float d3 = __uint_as_float(a.w) - __uint_as_float(b.w);
  return __builtin_fmaf(d3, d3, __builtin_fmaf(d2, d2, __builtin_fmaf(d1, d1, d0 * d0)));
}

// A 32-bit word holds two bfloat16; each widens exactly to float32 by a shift or a mask.
__device__ __forceinline__ float sqdiff_bf16x2(uint32_t a, uint32_t b) {
  const float lo = __uint_as_float(a << 16) - __uint_as_float(b << 16);
  const float hi = __uint_as_float(a & 0xffff0000u) - __uint_as_float(b & 0xffff0000u);
  return __builtin_fmaf(hi, hi, lo * lo);
}

__device__ __forceinline__ float sqdiff_bf16(const uint4& a, const uint4& b) {
  return (sqdiff_bf16x2(a.x, b.x) + sqdiff_bf16x2(a.y, b.y)) +
         (sqdiff_bf16x2(a.z, b.z) + sqdiff_bf16x2(a.w, b.w));
}

// Sums of absolute differences (total variation), added in a fixed order.
__device__ __forceinline__ float absdiff_f32(const uint4& a, const uint4& b) {
  const float d0 = __builtin_fabsf(__uint_as_float(a.x) - __uint_as_float(b.x));
  const float d1 = __builtin_fabsf(__uint_as_float(a.y) - __uint_as_float(b.y));
  const float d2 = __builtin_fabsf(__uint_as_float(a.z) - __uint_as_float(b.z));
  const float d3 = __builtin_fabsf(__uint_as_float(a.w) - __uint_as_float(b.w));
  return (d0 + d1) + (d2 + d3);
}

__device__ __forceinline__ float absdiff_bf16x2(uint32_t a, uint32_t b) {
  const float lo = __uint_as_float(a << 16) - __uint_as_float(b << 16);
  const float hi = __uint_as_float(a & 0xffff0000u) - __uint_as_float(b & 0xffff0000u);
  return __builtin_fabsf(lo) + __builtin_fabsf(hi);
}

__device__ __forceinline__ float absdiff_bf16(const uint4& a, const uint4& b) {
  return (absdiff_bf16x2(a.x, b.x) + absdiff_bf16x2(a.y, b.y)) +
         (absdiff_bf16x2(a.z, b.z) + absdiff_bf16x2(a.w, b.w));
}

// |a - b| of two int32 held in uint32: the true difference is below 2^32, so the
// unsigned subtraction of the smaller from the larger is exact.
__device__ __forceinline__ uint32_t absdiff_i32(uint32_t a, uint32_t b) {
  int32_t sa = (int32_t)a, sb = (int32_t)b;
  return sa > sb ? a - b : b - a;
}

__device__ __forceinline__ uint64_t absdiff_i32x4(const uint4& a, const uint4& b) {
  return (uint64_t)absdiff_i32(a.x, b.x) + absdiff_i32(a.y, b.y) + absdiff_i32(a.z, b.z) +
         absdiff_i32(a.w, b.w);
}

// ---- accumulators ------------------------------------------------------------------
// Float stores: each 16-byte step is summed in float32 and folded into a float64
// running sum, so long blocks and long index lists keep full accuracy.
// Integer stores: exact in uint64.

template <int DT>
struct Acc {
  using type = double;
};
template <>
struct Acc<DT_I32> {
  using type = unsigned long long;
};

template <int DT, int U>
__device__ __forceinline__ void accumulate_vec(typename Acc<DT>::type& acc, const uint4 (&a)[U],
                                               const uint4 (&b)[U]) {
  if constexpr (DT == DT_I32) {
#pragma unroll
    for (int u = 0; u < U; ++u) acc += absdiff_i32x4(a[u], b[u]);
  } else {
    float part = 0.f;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if constexpr (DT == DT_F32) part += sqdiff_f32(a[u], b[u]);
      if constexpr (DT == DT_BF16) part += sqdiff_bf16(a[u], b[u]);
      if constexpr (DT == DT_F32_TV) part += absdiff_f32(a[u], b[u]);
      if constexpr (DT == DT_BF16_TV) part += absdiff_bf16(a[u], b[u]);
    }
    acc += (double)part;
  }
}

template <int DT>
__device__ __forceinline__ void accumulate_elem(typename Acc<DT>::type& acc, const char* a,
                                                const char* b, uint64_t j) {
  if constexpr (DT == DT_I32) {
    acc += absdiff_i32(((const uint32_t*)a)[j], ((const uint32_t*)b)[j]);
  } else if constexpr (DT == DT_F32) {
    acc += (double)sq(((const float*)a)[j] - ((const float*)b)[j]);
  } else if constexpr (DT == DT_F32_TV) {
    acc += (double)__builtin_fabsf(((const float*)a)[j] - ((const float*)b)[j]);
  } else {
    uint32_t ua = ((const uint16_t*)a)[j], ub = ((const uint16_t*)b)[j];
    const float d = __uint_as_float(ua << 16) - __uint_as_float(ub << 16);
    acc += (double)(DT == DT_BF16 ? sq(d) : __builtin_fabsf(d));
  }
}

// ---- reductions --------------------------------------------------------------------

// Sum over the G lanes of a group (G a power of two <= 64); every lane gets the total.
template <int G, typename T>
__device__ __forceinline__ T group_sum(T v) {
#pragma unroll
  for (int m = G / 2; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
  return v;
}

// Sum over a workgroup of T threads; the result is valid in thread 0.  `slots` is LDS for
// T / kWave values.  Fixed order, so the result is reproducible.
template <int T = kWG, typename V>
__device__ __forceinline__ V workgroup_sum(V v, V* slots) {
  v = group_sum<kWave>(v);
  const int wave = threadIdx.x / kWave;
  __syncthreads();  // slots may still be read from a previous use
  if ((threadIdx.x & (kWave - 1)) == 0) slots[wave] = v;
  __syncthreads();
  V total = slots[0];
#pragma unroll
  for (int w = 1; w < T / kWave; ++w) total += slots[w];
  return total;
}

// Exclusive prefix sum of v over a workgroup of NT threads in thread order; *total gets the
// sum.  `slots` is LDS for NT / kWave + 1 values.
template <int NT = kWG, typename T>
__device__ __forceinline__ T workgroup_exclusive_scan(T v, T* slots, T* total) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  T inc = v;
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    T up = __shfl_up(inc, d, kWave);
    if (lane >= d) inc += up;
  }
  __syncthreads();
  if (lane == kWave - 1) slots[wave] = inc;
  __syncthreads();
  T base = 0, sum = 0;
#pragma unroll
  for (int w = 0; w < NT / kWave; ++w) {
    if (w < wave) base += slots[w];
    sum += slots[w];
  }
  *total = sum;
  return base + inc - v;
}

// ---- one block, one group ------------------------------------------------------------

// Geometry of block b: byte offset of its first element and its element count.
struct BlockSpan {
  uint64_t byte_off;
  uint32_t len;
};

__device__ __forceinline__ BlockSpan block_span(uint64_t b, uint64_t n_elems, uint32_t block_len,
                                                int ebytes) {
  uint64_t lo = b * (uint64_t)block_len;
  uint64_t hi = lo + block_len;
  if (hi > n_elems) hi = n_elems;
  return {lo * (uint64_t)ebytes, (uint32_t)(hi - lo)};
}

// How a row that need not start on a 16-byte boundary is walked: `head` single elements up
// to the next boundary, then `nvec` 16-byte steps, then the remaining elements.  The two
// streams must sit at the same offset within their 16-byte lines; if they do not, the whole
// row is walked element by element.  E = element size in bytes (pointers are E-aligned).
struct RowSplit {
  uint32_t head, nvec;
};

template <int E>
__device__ __forceinline__ RowSplit row_split(const void* a, const void* b, uint32_t len) {
  const uint32_t ma = (uint32_t)((uintptr_t)a & 15), mb = (uint32_t)((uintptr_t)b & 15);
  if (ma != mb) return {len, 0};
  uint32_t head = ((16 - ma) & 15) / E;
  if (head > len) head = len;
  return {head, (len - head) / (16 / E)};
}

// Distance term of one block, spread over the G lanes of a group; each lane returns its
// share.  VEC: every block of both streams starts 16-byte aligned and is a whole number of
// 16-byte steps; otherwise each row is split as row_split says.
template <int DT, int G, bool VEC>
__device__ __forceinline__ typename Acc<DT>::type block_distance(const char* xb, const char* cb,
                                                                 uint32_t len, int lane) {
  constexpr int E = elem_bytes(DT);
  constexpr int EPV = 16 / E;
  using word_t = typename std::conditional<E == 4, uint32_t, uint16_t>::type;
  typename Acc<DT>::type acc = 0;
  uint32_t head = 0, nvec;
  // The few elements before and after the 16-byte steps of a split row are asked for together
  // with the first steps (one round trip to memory less at each end of the row) when the group
  // has a lane for each of them; they are still added in the order head, steps, tail.
  bool has_head = false, has_tail = false;
  word_t hx = 0, hc = 0, tx = 0, tc = 0;
  if constexpr (VEC) {
    nvec = len / EPV;
  } else {
    const RowSplit rs = row_split<E>(xb, cb, len);
    head = rs.head, nvec = rs.nvec;
    if (G >= EPV && head < (uint32_t)EPV) {
      const uint32_t tail0 = head + nvec * EPV;
      has_head = (uint32_t)lane < head, has_tail = tail0 + lane < len;
      if (has_head) hx = ((const word_t*)xb)[lane], hc = ((const word_t*)cb)[lane];
      if (has_tail) tx = ((const word_t*)xb)[tail0 + lane], tc = ((const word_t*)cb)[tail0 + lane];
      if (nvec == 0 && has_head) accumulate_elem<DT>(acc, (const char*)&hx, (const char*)&hc, 0);
    } else {
      for (uint32_t j = lane; j < head; j += G) accumulate_elem<DT>(acc, xb, cb, j);
    }
  }
  const uint4* xv = (const uint4*)(xb + (size_t)head * E);
  const uint4* cv = (const uint4*)(cb + (size_t)head * E);
  for (uint32_t v0 = 0; v0 < nvec; v0 += G * kUnroll) {
    uint4 a[kUnroll], b[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      // a whole workgroup on a row: each wavefront takes kUnroll consecutive KiB of a round
      // rather than a KiB out of every fourth (measured faster, as for the scan of 4 KiB blocks)
      const uint32_t v = G == 256 ? v0 + ((lane / kWave) * kUnroll + u) * kWave + (lane & (kWave - 1))
                                  : v0 + u * G + lane;
      if (v < nvec) {
        a[u] = load_stream(xv + v);
        b[u] = load_stream(cv + v);
      } else {
        a[u] = make_uint4(0, 0, 0, 0);
        b[u] = make_uint4(0, 0, 0, 0);
      }
    }
    if constexpr (!VEC)
      if (v0 == 0 && has_head) accumulate_elem<DT>(acc, (const char*)&hx, (const char*)&hc, 0);
    accumulate_vec<DT, kUnroll>(acc, a, b);
  }
  if constexpr (!VEC) {
    if (G >= EPV && head < (uint32_t)EPV) {
      if (has_tail) accumulate_elem<DT>(acc, (const char*)&tx, (const char*)&tc, 0);
      return acc;
    }
  }
  for (uint32_t j = head + nvec * EPV + lane; j < len; j += G) accumulate_elem<DT>(acc, xb, cb, j);
  return acc;
}

// The 16-byte steps of a copy: kUnroll loads per lane, then the stores.
template <int G>
__device__ __forceinline__ void copy_steps(const uint4* s, uint4* d, uint4* d2, uint32_t nvec, int lane) {
  for (uint32_t v0 = 0; v0 < nvec; v0 += G * kUnroll) {
    uint4 a[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const uint32_t v = v0 + u * G + lane;
      a[u] = v < nvec ? load_stream(s + v) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const uint32_t v = v0 + u * G + lane;
      if (v < nvec) {
        store_stream(d + v, a[u]);
        if (d2) store_stream(d2 + v, a[u]);
      }
    }
  }
}

// Copy one block src -> dst (and to dst2 if not NULL), spread over a group.  W is the
// word type of the element-wise path (uint32_t for 4-byte elements, uint16_t for 2-byte).
// vec: src and dst start 16-byte aligned; otherwise the row is split as row_split says.
// vec2 (only with vec): dst2 can take the same 16-byte steps.
// The few elements before and after the 16-byte steps of a split row are fetched together
// with the first steps - one round trip to memory for a short row, not three (when the group
// has a lane for each of them: G >= 16 / sizeof(W)).
template <int G, typename W>
__device__ __forceinline__ void block_copy(const char* src, char* dst, char* dst2, uint32_t nbytes,
                                           int lane, bool vec, bool vec2) {
  constexpr uint32_t WPV = 16 / sizeof(W);
  const uint32_t nword = nbytes / sizeof(W);
  const W* sw = (const W*)src;
  W* dw = (W*)dst;
  if (vec) {  // whole steps, and a tail that only the store's short last block has
    const uint32_t nvec = nbytes / 16;
    copy_steps<G>((const uint4*)src, (uint4*)dst, (dst2 && vec2) ? (uint4*)dst2 : nullptr, nvec, lane);
    for (uint32_t h = nvec * WPV + lane; h < nword; h += G) dw[h] = sw[h];
    if (dst2)
      for (uint32_t h = (vec2 ? nvec * WPV : 0) + lane; h < nword; h += G) ((W*)dst2)[h] = sw[h];
    return;
  }
  const RowSplit rs = row_split<sizeof(W)>(src, dst, nword);
  const uint32_t head = rs.head, nvec = rs.nvec, tail0 = head + nvec * WPV;
  const bool ends_in_lanes = G >= WPV && head < WPV;  // else: a row walked element by element
  W hw = 0, tw = 0;
  if (ends_in_lanes) {
    if ((uint32_t)lane < head) hw = sw[lane];
    if (tail0 + lane < nword) tw = sw[tail0 + lane];
  } else {
    for (uint32_t h = lane; h < head; h += G) dw[h] = sw[h];
  }
  const uint4* s = (const uint4*)(src + (size_t)head * sizeof(W));
  uint4* d = (uint4*)(dst + (size_t)head * sizeof(W));
  if (ends_in_lanes && nvec <= (uint32_t)G * kUnroll) {
    // a short row: everything is asked for before anything is stored, and the stores go out
    // in address order (measured faster than the head after the steps: 100-byte rows 235 vs 280 us)
    uint4 a[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const uint32_t v = u * G + lane;
      a[u] = v < nvec ? load_stream(s + v) : make_uint4(0, 0, 0, 0);
    }
    if ((uint32_t)lane < head) dw[lane] = hw;
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const uint32_t v = u * G + lane;
      if (v < nvec) store_stream(d + v, a[u]);
    }
    if (tail0 + lane < nword) dw[tail0 + lane] = tw;
  } else {
    if (ends_in_lanes && (uint32_t)lane < head) dw[lane] = hw;
    copy_steps<G>(s, d, nullptr, nvec, lane);
    if (ends_in_lanes) {
      if (tail0 + lane < nword) dw[tail0 + lane] = tw;
    } else {
      for (uint32_t h = tail0 + lane; h < nword; h += G) dw[h] = sw[h];
    }
  }
  if (dst2)  // rows of the staging buffer are packed: no 16-byte steps that match the source's
    for (uint32_t h = lane; h < nword; h += G) ((W*)dst2)[h] = sw[h];
}

}  // namespace scar
