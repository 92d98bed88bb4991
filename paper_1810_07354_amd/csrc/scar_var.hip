// Blocks of unequal length (Section 5.1: "by-layer" partitioning, every weight or bias
// tensor one parameter): scar_var_block_scores, scar_var_checkpoint_commit,
// scar_var_partial_recover, scar_var_perturbation_norm.
//
// Block b is the element range [offsets[b], offsets[b+1]).  Sizes can differ by orders of
// magnitude (a 3-million-element matrix next to a 10-element bias), so work is not dealt
// out by block but by position: the store is cut into equal ranges of consecutive
// elements, one workgroup per range.  A small planning kernel finds, for every range, the
// block that holds its first element (binary search over the offsets) and whether the range
// touches a chosen block at all; a workgroup then walks forward through its range, segment
// by segment, where a segment is the part of one block that lies inside the range.
//
//   scores:  the workgroup's sum for block b goes to partial[w + b] (w = range number).
//            Along the store either w or b grows from one (range, block) pair to the next,
//            so the slots are distinct and those of one block are consecutive; a second
//            kernel adds each block's slots in a fixed order.  A giant block is thus summed
//            by as many workgroups as it spans, a run of tiny blocks by one.
//   commit / recover / norm:  a byte per block marks the chosen ones; every workgroup
//            handles the chosen segments of its range and skips the rest (ranges without a
//            chosen block leave at once).  Here ranges go to the XCDs round-robin, because a
//            chosen tensor is one contiguous stretch and must not land on a single XCD; the
//            dense score walk gives each XCD a contiguous eighth instead.
//
//   packed rows (the storage leg, Section 4.3): a commit can also pack the chosen blocks one
//            after the other, in list order, into a staging buffer, and a recovery can take the
//            checkpoint values from such packed rows instead of from c.  pack[b] holds the
//            element offset of block b in the packed buffer (a prefix sum over the list for a
//            commit, the caller's row offsets for a recovery); the packed side of a segment
//            starts wherever the lengths before it add up to, so it is read and written in
//            4-byte (2-byte) words next to the 16-byte accesses of x and c.
//
// Segments start wherever a block starts, so each is split into a few leading elements up
// to the next 16-byte boundary, a body of non-temporal 16-byte accesses, and a tail.
#include "scar_device.hpp"
#include "scar_host.hpp"
#include "scar_mixed_device.hpp"

namespace scar {

// Planning of range w: first[w] = the block that holds the range's first element
// (offsets[b] <= e < offsets[b+1]); any[w] = 1 if a block with mask != 0 reaches into the
// range (always 1 without a mask).  Whatever the offsets hold, first[w] < n_blocks.
__device__ __forceinline__ void plan_range(uint32_t w, const uint64_t* __restrict__ off, uint32_t n_blocks,
                                           uint64_t n_elems, uint64_t range_elems, const uint8_t* mask,
                                           uint32_t* __restrict__ first, uint8_t* __restrict__ any) {
  const uint64_t e0 = (uint64_t)w * range_elems;
  const uint64_t e1 = e0 + range_elems < n_elems ? e0 + range_elems : n_elems;
  uint32_t lo = 0, hi = n_blocks;
  while (hi - lo > 1) {
    const uint32_t mid = lo + (hi - lo) / 2;
    if (off[mid] <= e0)
      lo = mid;
    else
      hi = mid;
  }
  first[w] = lo;
  uint8_t hit = mask ? 0 : 1;
  if (mask) {
    for (uint32_t b = lo; b < n_blocks && off[b] < e1; ++b) {
      if (mask[b] && off[b + 1] > off[b] && off[b + 1] > e0) {
        hit = 1;
        break;
      }
    }
  }
  any[w] = hit;
}

// One thread per range.
__global__ __launch_bounds__(kWG) void k_var_plan(const uint64_t* __restrict__ off, uint32_t n_blocks,
                                                  uint64_t n_elems, uint64_t range_elems, uint32_t n_wg,
                                                  const uint8_t* __restrict__ mask,
                                                  uint32_t* __restrict__ first, uint8_t* __restrict__ any) {
  const uint32_t w = blockIdx.x * kWG + threadIdx.x;
  if (w < n_wg) plan_range(w, off, n_blocks, n_elems, range_elems, mask, first, any);
}

// Small stores (few ranges, few blocks - a network cut by layer): marking the chosen blocks
// and planning the ranges in one launch by one workgroup instead of three launches.
constexpr int kPrepareThreads = 1024;
constexpr uint32_t kPrepareMaxRanges = 1024;
constexpr uint32_t kPrepareMaxBlocks = 65536;
__global__ __launch_bounds__(kPrepareThreads) void k_var_prepare(
    const uint64_t* __restrict__ off, uint32_t n_blocks, uint64_t n_elems, uint64_t range_elems,
    uint32_t n_wg, uint8_t* mask, const uint32_t* __restrict__ idx, uint32_t n_idx,
    uint32_t* __restrict__ first, uint8_t* __restrict__ any) {
  for (uint32_t b = threadIdx.x; b < n_blocks; b += kPrepareThreads) mask[b] = 0;
  __syncthreads();
  for (uint32_t i = threadIdx.x; i < n_idx; i += kPrepareThreads) {
    const uint32_t b = idx[i];
    if (b < n_blocks) mask[b] = 1;
  }
  __syncthreads();
  for (uint32_t w = threadIdx.x; w < n_wg; w += kPrepareThreads)
    plan_range(w, off, n_blocks, n_elems, range_elems, mask, first, any);
}

enum : int { COPY_NONE = 0, COPY_X_TO_C = 1, COPY_C_TO_X = 2 };
// What the packed side buffer does: nothing, receive the segment as well (staging rows of a
// commit), or stand in for c (rows read back from storage).
enum : int { SIDE_NONE = 0, SIDE_WRITE = 1, SIDE_READ = 2 };

// 16 bytes of a buffer that is only element-aligned, as words.
template <typename W>
__device__ __forceinline__ uint4 load_words(const W* p) {
  constexpr int N = 16 / sizeof(W);
  W w[N];
#pragma unroll
  for (int i = 0; i < N; ++i) w[i] = p[i];
  uint4 v;
  __builtin_memcpy(&v, w, 16);
  return v;
}
template <typename W>
__device__ __forceinline__ void store_words(W* p, const uint4& v) {
  constexpr int N = 16 / sizeof(W);
  W w[N];
  __builtin_memcpy(w, &v, 16);
#pragma unroll
  for (int i = 0; i < N; ++i) p[i] = w[i];
}

// A segment of a float32 store with a bfloat16 checkpoint (SCAR_F32_BF16C): the unit is 4
// elements, 16 bytes of x against 8 bytes of c; a commit stores x rounded to nearest even (and
// the same rounded values in the staging rows), a recovery widens.  `side` is only 2-byte
// aligned and is read and written in halfwords.
template <bool ACC, int COPY, int SIDE>
__device__ __forceinline__ void segment_apply_mixed(float* __restrict__ x, uint16_t* __restrict__ c,
                                                    uint16_t* __restrict__ side, uint64_t first, uint64_t len,
                                                    bool base_aligned, double& acc) {
  float* xs = x + first;
  uint16_t* cs = SIDE == SIDE_READ ? side : c + first;
  auto element = [&](uint64_t j) {
    if (ACC) acc += (double)sq(xs[j] - widen_elem(cs, j));
    if (COPY == COPY_X_TO_C) {
      const uint16_t r = (uint16_t)round_bf16(__float_as_uint(xs[j]));
      cs[j] = r;
      if (SIDE == SIDE_WRITE) side[j] = r;
    }
    if (COPY == COPY_C_TO_X) xs[j] = widen_elem(cs, j);
  };
  uint64_t head = len;  // elements handled one by one before the whole units
  if (base_aligned) {
    head = (kMixUnit - (first & (kMixUnit - 1))) & (kMixUnit - 1);
    if (head > len) head = len;
  }
  for (uint64_t j = threadIdx.x; j < head; j += kWG) element(j);
  const uint64_t nunit = (len - head) / kMixUnit;
  uint4* xv = (uint4*)(xs + head);
  uint2* cv = (uint2*)(cs + head);  // SIDE_READ: only 2-byte aligned, read in halfwords below
  constexpr int U = COPY == COPY_NONE ? kMixU : 2;
  for (uint64_t v0 = 0; v0 < nunit; v0 += (uint64_t)kWG * U) {
    uint4 a[U];
    uint2 b[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint64_t v = v0 + (uint64_t)u * kWG + threadIdx.x;
      const bool ok = v < nunit;
      a[u] = (ok && (ACC || COPY == COPY_X_TO_C)) ? load_stream(xv + v) : make_uint4(0, 0, 0, 0);
      b[u] = make_uint2(0, 0);
      if (ok && (ACC || COPY == COPY_C_TO_X)) {
        if (SIDE == SIDE_READ) {
          const uint16_t* h = cs + head + v * kMixUnit;
          b[u] = make_uint2((uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16));
        } else {
          b[u] = load_stream2(cv + v);
        }
      }
    }
    if (ACC) {
      float part = 0.f;
#pragma unroll
      for (int u = 0; u < U; ++u) part += sqdiff_unit(a[u], b[u]);
      acc += (double)part;
    }
    if (COPY != COPY_NONE) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint64_t v = v0 + (uint64_t)u * kWG + threadIdx.x;
        if (v >= nunit) continue;
        if (COPY == COPY_X_TO_C) {
          const uint2 r = round_unit(a[u]);
          store_stream2(cv + v, r);
          if (SIDE == SIDE_WRITE) {
            uint16_t* h = side + head + v * kMixUnit;
            h[0] = (uint16_t)r.x, h[1] = (uint16_t)(r.x >> 16), h[2] = (uint16_t)r.y, h[3] = (uint16_t)(r.y >> 16);
          }
        }
        if (COPY == COPY_C_TO_X) store_stream(xv + v, widen_unit(b[u]));
      }
    }
  }
  for (uint64_t j = head + nunit * kMixUnit + threadIdx.x; j < len; j += kWG) element(j);
}

// One segment of `len` elements starting at element `first`, spread over the workgroup.
//   ACC:  acc += sum of (c - x)^2 or |c - x| over the segment (this lane's share)
//   COPY: the segment is copied x -> c or c -> x afterwards
//   SIDE: `side` points at the segment's place in the packed buffer (element-aligned):
//         SIDE_WRITE stores the segment of x there too, SIDE_READ takes c's values from there
//         (c itself is then not touched).
template <int DT, bool ACC, int COPY, int SIDE>
__device__ __forceinline__ void segment_apply(char* __restrict__ x, char* __restrict__ c,
                                              char* __restrict__ side, uint64_t first, uint64_t len,
                                              bool base_aligned, typename Acc<DT>::type& acc) {
  if constexpr (DT == DT_MIXED) {
    segment_apply_mixed<ACC, COPY, SIDE>((float*)x, (uint16_t*)c, (uint16_t*)side, first, len, base_aligned, acc);
    return;
  }
  constexpr int E = elem_bytes(DT);
  constexpr int EPV = 16 / E;
  using word_t = typename std::conditional<E == 4, uint32_t, uint16_t>::type;
  char* xs = x + first * E;
  char* cs = SIDE == SIDE_READ ? side : c + first * E;
  auto element = [&](uint64_t j) {
    if (ACC) accumulate_elem<DT>(acc, cs, xs, j);
    if (COPY == COPY_X_TO_C) ((word_t*)cs)[j] = ((const word_t*)xs)[j];
    if (COPY == COPY_C_TO_X) ((word_t*)xs)[j] = ((const word_t*)cs)[j];
    if (SIDE == SIDE_WRITE) ((word_t*)side)[j] = ((const word_t*)xs)[j];
  };
  uint64_t head = len;  // elements handled one by one before the 16-byte body
  if (base_aligned) {
    head = ((16 - ((first * E) & 15)) & 15) / E;
    if (head > len) head = len;
  }
  for (uint64_t j = threadIdx.x; j < head; j += kWG) element(j);
  const uint64_t nvec = (len - head) / EPV;
  uint4* xv = (uint4*)(xs + head * E);
  uint4* cv = (uint4*)(cs + head * E);          // SIDE_READ: only element-aligned, see below
  word_t* sw = (word_t*)(side + (SIDE == SIDE_NONE ? 0 : head * E));
  // a pure read keeps four loads per lane and stream in flight; copies do best with fewer
  constexpr int U = COPY == COPY_NONE ? kUnroll : 2;
  for (uint64_t v0 = 0; v0 < nvec; v0 += (uint64_t)kWG * U) {
    uint4 a[U], b[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint64_t v = v0 + (uint64_t)u * kWG + threadIdx.x;
      const bool ok = v < nvec;
      a[u] = (ok && (ACC || COPY == COPY_X_TO_C)) ? load_stream(xv + v) : make_uint4(0, 0, 0, 0);
      if (SIDE == SIDE_READ)
        b[u] = ok ? load_words((const word_t*)cs + (head + v * EPV)) : make_uint4(0, 0, 0, 0);
      else
        b[u] = (ok && (ACC || COPY == COPY_C_TO_X)) ? load_stream(cv + v) : make_uint4(0, 0, 0, 0);
    }
    if (ACC) accumulate_vec<DT, U>(acc, b, a);
    if (COPY != COPY_NONE) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint64_t v = v0 + (uint64_t)u * kWG + threadIdx.x;
        if (v < nvec) {
          if (COPY == COPY_X_TO_C) store_stream(cv + v, a[u]);
          if (COPY == COPY_C_TO_X) store_stream(xv + v, b[u]);
          if (SIDE == SIDE_WRITE) store_words(sw + v * EPV, a[u]);
        }
      }
    }
  }
  for (uint64_t j = head + nvec * EPV + threadIdx.x; j < len; j += kWG) element(j);
}

// The walk over one range.
//   PER_BLOCK (scores): every block met gets its own sum in partial[w + b].
//   otherwise: only blocks with mask[b] != 0 (all blocks if mask == NULL) are touched and
//   the workgroup's total goes to partial[w] (if ACC).
//   SIDE: the packed buffer `side` with the per-block element offsets `pack` (see above).
template <int DT, bool ACC, int COPY, bool PER_BLOCK, int SIDE>
__global__ __launch_bounds__(kWG) void k_var_walk(char* __restrict__ x, char* __restrict__ c,
                                                  const uint64_t* __restrict__ off, uint32_t n_blocks,
                                                  uint64_t n_elems, uint64_t range_elems, uint32_t n_wg,
                                                  const uint8_t* __restrict__ mask,
                                                  const uint32_t* __restrict__ first,
                                                  const uint8_t* __restrict__ any,
                                                  typename Acc<DT>::type* __restrict__ partial,
                                                  bool base_aligned, char* __restrict__ side,
                                                  const uint64_t* __restrict__ pack,
                                                  const float* __restrict__ weights) {
  using acc_t = typename Acc<DT>::type;
  __shared__ acc_t slots[kWG / kWave];
  const uint32_t w = PER_BLOCK ? xcd_contiguous_block_id() : blockIdx.x;
  if (w >= n_wg) return;
  if (!PER_BLOCK && !any[w]) {  // nothing chosen in this range
    if (ACC && threadIdx.x == 0) partial[w] = 0;
    return;
  }
  const uint64_t e0 = (uint64_t)w * range_elems;
  const uint64_t e1 = e0 + range_elems < n_elems ? e0 + range_elems : n_elems;
  uint32_t cur = first[w];
  acc_t acc = 0;
  uint64_t pos = e0;
  while (pos < e1) {
    uint64_t bend = off[cur + 1];
    while (bend <= pos && cur + 1 < n_blocks) {  // block `cur` ends here: hand in its sum
      if (PER_BLOCK) {
        const acc_t total = workgroup_sum(acc, slots);
        if (threadIdx.x == 0) partial[(uint64_t)w + cur] = total;
        acc = 0;
      }
      ++cur;
      bend = off[cur + 1];
    }
    if (bend <= pos) break;  // offsets do not cover the store: leave the rest alone
    const uint64_t seg_end = bend < e1 ? bend : e1;
    if (PER_BLOCK || !mask || mask[cur]) {
      char* side_seg = nullptr;
      if constexpr (SIDE != SIDE_NONE) side_seg = side + (pack[cur] + (pos - off[cur])) * c_elem_bytes(DT);
      if constexpr (is_tv(DT) && ACC && !PER_BLOCK) {  // a row's share counts with the row's weight
        const float w = weights ? weights[cur] : 1.f;
        acc_t seg = 0;
        segment_apply<DT, ACC, COPY, SIDE>(x, c, side_seg, pos, seg_end - pos, base_aligned, seg);
        acc += (double)w * seg;
      } else {
        segment_apply<DT, ACC, COPY, SIDE>(x, c, side_seg, pos, seg_end - pos, base_aligned, acc);
      }
    }
    pos = seg_end;
  }
  if (ACC) {
    const acc_t total = workgroup_sum(acc, slots);
    if (threadIdx.x == 0) partial[PER_BLOCK ? (uint64_t)w + cur : (uint64_t)w] = total;
  }
}

// Second stage of the scores: G lanes (of a workgroup of T threads; G = T or G <= 64) add the
// slots of one block in a fixed order.
template <int DT, int G, int T>
__global__ __launch_bounds__(T) void k_var_scores_finish(const typename Acc<DT>::type* __restrict__ partial,
                                                         const uint64_t* __restrict__ off,
                                                         uint32_t n_blocks, uint64_t n_elems,
                                                         uint64_t range_elems, void* __restrict__ scores,
                                                         const float* __restrict__ weights) {
  using acc_t = typename Acc<DT>::type;
  constexpr int GPW = T / G;
  __shared__ acc_t slots[T / kWave];
  const int lane = threadIdx.x & (G - 1);
  for (uint64_t b = (uint64_t)blockIdx.x * GPW + threadIdx.x / G; b < n_blocks;
       b += (uint64_t)gridDim.x * GPW) {
    const uint64_t lo = off[b];
    uint64_t hi = off[b + 1];
    if (hi > n_elems) hi = n_elems;
    acc_t acc = 0;
    if (hi > lo) {
      const uint64_t w_first = lo / range_elems, w_last = (hi - 1) / range_elems;
      const acc_t* slot = partial + w_first + b;
      const uint64_t n_slots = w_last - w_first + 1;
      uint64_t i = lane;
      for (; i + 7 * G < n_slots; i += 8 * G) {  // eight loads in flight, added in index order
        acc_t t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) t[u] = slot[i + u * G];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += t[u];
      }
      for (; i < n_slots; i += G) acc += slot[i];
    }
    if constexpr (G == T)
      acc = workgroup_sum<T>(acc, slots);
    else
      acc = group_sum<G>(acc);
    if (lane == 0) {
      if constexpr (DT == DT_I32)
        ((long long*)scores)[b] = (long long)acc;
      else if constexpr (is_tv(DT))  // w_b * 1/2 * sum |x - c|
        ((float*)scores)[b] = (float)(0.5 * acc * (double)(weights ? weights[b] : 1.f));
      else
        ((float*)scores)[b] = (float)acc;
    }
  }
}

__global__ __launch_bounds__(kWG) void k_var_mask_clear(uint8_t* __restrict__ mask, uint32_t n_blocks) {
  for (uint64_t i = (uint64_t)blockIdx.x * kWG + threadIdx.x; i < n_blocks; i += (uint64_t)gridDim.x * kWG)
    mask[i] = 0;
}

__global__ __launch_bounds__(kWG) void k_var_mask_set(uint8_t* __restrict__ mask, uint32_t n_blocks,
                                                      const uint32_t* __restrict__ idx, uint32_t n_idx) {
  for (uint64_t i = (uint64_t)blockIdx.x * kWG + threadIdx.x; i < n_idx; i += (uint64_t)gridDim.x * kWG) {
    const uint32_t b = idx[i];
    if (b < n_blocks) mask[b] = 1;
  }
}

// Packed offsets of a commit with staging rows: out[i] = elements of the blocks listed before
// idx[i] (out[n_idx] = all of them), and pack[idx[i]] = out[i].  One workgroup; entries
// >= n_blocks take no room.
constexpr int kPackThreads = 1024;
__global__ __launch_bounds__(kPackThreads) void k_var_pack_scan(const uint64_t* __restrict__ off,
                                                                uint32_t n_blocks,
                                                                const uint32_t* __restrict__ idx, uint32_t n_idx,
                                                                unsigned long long* __restrict__ out,
                                                                unsigned long long* __restrict__ pack) {
  __shared__ unsigned long long slots[kPackThreads / kWave + 1];
  unsigned long long running = 0;
  for (uint32_t i0 = 0; i0 < n_idx; i0 += kPackThreads) {
    const uint32_t i = i0 + threadIdx.x;
    const uint32_t b = i < n_idx ? idx[i] : n_blocks;
    const unsigned long long len = b < n_blocks ? off[b + 1] - off[b] : 0ull;
    unsigned long long total;
    const unsigned long long ex = workgroup_exclusive_scan<kPackThreads>(len, slots, &total);
    if (i < n_idx) out[i] = running + ex;
    if (b < n_blocks) pack[b] = running + ex;
    running += total;
    __syncthreads();
  }
  if (threadIdx.x == 0) out[n_idx] = running;
}

// Packed offsets of a recovery from rows: pack[lost[i]] = row_offsets[i].
__global__ __launch_bounds__(kWG) void k_var_pack_set(uint32_t n_blocks, const uint32_t* __restrict__ idx,
                                                      uint32_t n_idx, const uint64_t* __restrict__ row_offsets,
                                                      unsigned long long* __restrict__ pack) {
  for (uint64_t i = (uint64_t)blockIdx.x * kWG + threadIdx.x; i < n_idx; i += (uint64_t)gridDim.x * kWG) {
    const uint32_t b = idx[i];
    if (b < n_blocks) pack[b] = row_offsets[i];
  }
}

static uint64_t var_blocks(const scar_var_layout* l) {
  if (!l || !dtype_ok(l->dtype) || l->n_blocks > SCAR_MAX_BLOCKS) return UINT64_MAX;
  if (l->n_blocks && (!l->offsets || !aligned(l->offsets, 8))) return UINT64_MAX;
  return l->n_blocks;
}

static int check_var_workspace(const void* ws, size_t bytes, uint64_t n_blocks) {
  if (!ws || !aligned(ws, 256) || bytes < var_workspace_bytes_for(n_blocks)) return SCAR_ERR_WORKSPACE;
  return SCAR_OK;
}

template <int DT, bool ACC, int COPY, bool PER_BLOCK, int SIDE = SIDE_NONE>
static void launch_walk(const scar_var_layout* l, const void* x, const void* c, const uint8_t* mask,
                        bool planned, void* workspace, const VarGeometry& g, hipStream_t st,
                        void* side = nullptr, const float* weights = nullptr) {
  const bool base_aligned = aligned(x, 16) && aligned(c, DT == DT_MIXED ? 8 : 16);
  uint32_t* first = (uint32_t*)workspace;
  uint8_t* any = (uint8_t*)workspace + kVarPlanAnyOffset;
  void* partial = (char*)workspace + kVarPartialOffset;
  if (!planned)
    launch(k_var_plan, dim3((g.n_wg + kWG - 1) / kWG), dim3(kWG), 0, st, l->offsets, l->n_blocks,
                       l->n_elems, g.range_elems, g.n_wg, mask, first, any);
  // the score walk reads everything and keeps kUnroll 16-byte steps per lane and stream in flight
  uint64_t in_flight = 2 * g.range_elems * elem_bytes(DT);
  if (in_flight > 2 * 16 * kWG * kUnroll) in_flight = 2 * 16 * kWG * kUnroll;
  const size_t lds = (COPY == COPY_NONE && PER_BLOCK) ? stream_lds_bytes(g.n_wg, in_flight) : 0;
  const uint64_t* pack = (const uint64_t*)((char*)workspace + var_pack_offset(l->n_blocks));
  launch((k_var_walk<DT, ACC, COPY, PER_BLOCK, SIDE>), dim3(xcd_grid(g.n_wg, kVarMaxGridCopy)), dim3(kWG),
                     lds, st, (char*)const_cast<void*>(x), (char*)const_cast<void*>(c), l->offsets,
                     l->n_blocks, l->n_elems, g.range_elems, g.n_wg, mask, (const uint32_t*)first,
                     (const uint8_t*)any, (typename Acc<DT>::type*)partial, base_aligned, (char*)side, pack, weights);
}

template <bool ACC, int COPY, bool PER_BLOCK, int SIDE = SIDE_NONE>
static void dispatch_walk(const scar_var_layout* l, const void* x, const void* c, const uint8_t* mask,
                          bool planned, void* workspace, const VarGeometry& g, hipStream_t st,
                          void* side = nullptr) {
  switch (l->dtype) {
    case SCAR_F32: launch_walk<DT_F32, ACC, COPY, PER_BLOCK, SIDE>(l, x, c, mask, planned, workspace, g, st, side); break;
    case SCAR_BF16: launch_walk<DT_BF16, ACC, COPY, PER_BLOCK, SIDE>(l, x, c, mask, planned, workspace, g, st, side); break;
    case SCAR_F32_BF16C: launch_walk<DT_MIXED, ACC, COPY, PER_BLOCK, SIDE>(l, x, c, mask, planned, workspace, g, st, side); break;
    default: launch_walk<DT_I32, ACC, COPY, PER_BLOCK, SIDE>(l, x, c, mask, planned, workspace, g, st, side); break;
  }
}

// The total-variation kinds (float stores only; always measuring).
template <int COPY, bool PER_BLOCK>
static void dispatch_walk_tv(const scar_var_layout* l, const void* x, const void* c, const uint8_t* mask,
                             bool planned, void* workspace, const VarGeometry& g, const float* weights,
                             hipStream_t st) {
  if (l->dtype == SCAR_F32)
    launch_walk<DT_F32_TV, true, COPY, PER_BLOCK>(l, x, c, mask, planned, workspace, g, st, nullptr, weights);
  else
    launch_walk<DT_BF16_TV, true, COPY, PER_BLOCK>(l, x, c, mask, planned, workspace, g, st, nullptr, weights);
}

template <int DT>
static void launch_scores_finish(const scar_var_layout* l, const void* workspace, const VarGeometry& g,
                                 void* scores, hipStream_t st, const float* weights = nullptr) {
  using acc_t = typename Acc<DT>::type;
  const void* partial = (const char*)workspace + kVarPartialOffset;
  if (l->n_blocks <= 16384) {  // few blocks, possibly huge: a whole workgroup adds each one's slots
    launch((k_var_scores_finish<DT, 1024, 1024>), dim3(l->n_blocks), dim3(1024), 0, st,
                       (const acc_t*)partial, l->offsets, l->n_blocks, l->n_elems, g.range_elems, scores, weights);
  } else {
    const uint64_t need = ((uint64_t)l->n_blocks + 3) / 4;
    launch((k_var_scores_finish<DT, kWave, kWG>), dim3((uint32_t)(need < 65536 ? need : 65536)),
                       dim3(kWG), 0, st, (const acc_t*)partial, l->offsets, l->n_blocks, l->n_elems,
                       g.range_elems, scores, weights);
  }
}

// Marks the blocks of idx in the workspace's selection bytes; returns their address.  Small
// stores also get their ranges planned in the same launch (*planned = true).
static const uint8_t* mark_blocks(const scar_var_layout* l, const uint32_t* idx, uint32_t n_idx,
                                  void* workspace, const VarGeometry& g, bool* planned, hipStream_t st) {
  uint8_t* mask = (uint8_t*)workspace + var_mask_offset(l->n_blocks);
  if (g.n_wg <= kPrepareMaxRanges && l->n_blocks <= kPrepareMaxBlocks) {
    launch(k_var_prepare, dim3(1), dim3(kPrepareThreads), 0, st, l->offsets, l->n_blocks,
                       l->n_elems, g.range_elems, g.n_wg, mask, idx, n_idx, (uint32_t*)workspace,
                       (uint8_t*)workspace + kVarPlanAnyOffset);
    *planned = true;
    return mask;
  }
  const uint32_t cg = (l->n_blocks + kWG * 16 - 1) / (kWG * 16);
  launch(k_var_mask_clear, dim3(cg < 4096 ? cg : 4096), dim3(kWG), 0, st, mask, l->n_blocks);
  const uint32_t sg = (n_idx + kWG - 1) / kWG;
  launch(k_var_mask_set, dim3(sg < 4096 ? sg : 4096), dim3(kWG), 0, st, mask, l->n_blocks, idx,
                     n_idx);
  *planned = false;
  return mask;
}

// Shared body of commit (copy = COPY_X_TO_C), recovery (COPY_C_TO_X) and norm (COPY_NONE).
//   side / side_offsets: the packed buffer of a commit with staging rows (side_offsets is then
//   an output, n_idx + 1 entries) or of a recovery from rows (side_offsets is an input,
//   n_idx entries); both NULL otherwise.
static int var_rows(int copy, const scar_var_layout* layout, const void* x, const void* c,
                    const uint32_t* idx, uint32_t n_idx, bool all_blocks, scar_norm* norm_out,
                    void* workspace, size_t workspace_bytes, void* stream, void* side = nullptr,
                    uint64_t* side_offsets = nullptr, bool tv = false, const float* weights = nullptr) {
  if (tv && layout && (layout->dtype == SCAR_I32 || layout->dtype == SCAR_F32_BF16C)) return SCAR_ERR_UNSUPPORTED;
  if (!aligned(weights, 4)) return SCAR_ERR_INVALID_ARG;
  const uint64_t nb = var_blocks(layout);
  if (nb == UINT64_MAX) return SCAR_ERR_INVALID_ARG;
  if (norm_out && !aligned(norm_out, 8)) return SCAR_ERR_INVALID_ARG;
  const int rc = check_var_workspace(workspace, workspace_bytes, nb);
  if (rc) return rc;
  hipStream_t st = (hipStream_t)stream;
  const bool nothing = nb == 0 || layout->n_elems == 0 || (!all_blocks && n_idx == 0);
  if (side && (!side_offsets || !aligned(side_offsets, 8) || !aligned(side, host_c_elem_bytes(layout->dtype))))
    return SCAR_ERR_INVALID_ARG;
  if (nothing) {
    if (side && copy == COPY_X_TO_C)  // an empty list still gets its (all zero) offsets
      launch(k_var_pack_scan, dim3(1), dim3(kPackThreads), 0, st, layout->offsets, (uint32_t)nb, idx, 0u,
             (unsigned long long*)side_offsets, (unsigned long long*)((char*)workspace + var_pack_offset(nb)));
    if (norm_out) {
      if (tv)
        launch_finish_tv((char*)workspace + kVarPartialOffset, 0, norm_out, st);
      else
        launch_finish(layout->dtype, (char*)workspace + kVarPartialOffset, 0, norm_out, st);
    }
    return launch_status();
  }
  const int eb = host_elem_bytes(layout->dtype), ceb = host_c_elem_bytes(layout->dtype);
  if (!x || !c || (!all_blocks && !idx) || !aligned(x, eb) || !aligned(c, side && copy == COPY_C_TO_X ? eb : ceb) ||
      !aligned(idx, 4))
    return SCAR_ERR_INVALID_ARG;
  // walks that add nothing up take the finer cut
  const VarGeometry g = var_geometry(layout->n_elems, norm_out ? kVarMaxGrid : kVarMaxGridCopy);
  bool planned = false;
  const uint8_t* mask = all_blocks ? nullptr : mark_blocks(layout, idx, n_idx, workspace, g, &planned, st);
  unsigned long long* pack = (unsigned long long*)((char*)workspace + var_pack_offset(nb));
  if (side && copy == COPY_X_TO_C) {
    launch(k_var_pack_scan, dim3(1), dim3(kPackThreads), 0, st, layout->offsets, (uint32_t)nb, idx, n_idx,
           (unsigned long long*)side_offsets, pack);
    dispatch_walk<false, COPY_X_TO_C, false, SIDE_WRITE>(layout, x, c, mask, planned, workspace, g, st, side);
  } else if (side) {  // recovery from packed rows: c is not read
    const uint32_t sg = (n_idx + kWG - 1) / kWG;
    launch(k_var_pack_set, dim3(sg < 4096 ? sg : 4096), dim3(kWG), 0, st, (uint32_t)nb, idx, n_idx,
           (const uint64_t*)side_offsets, pack);
    if (norm_out)
      dispatch_walk<true, COPY_C_TO_X, false, SIDE_READ>(layout, x, x, mask, planned, workspace, g, st, side);
    else
      dispatch_walk<false, COPY_C_TO_X, false, SIDE_READ>(layout, x, x, mask, planned, workspace, g, st, side);
  } else if (tv && norm_out && copy == COPY_C_TO_X)
    dispatch_walk_tv<COPY_C_TO_X, false>(layout, x, c, mask, planned, workspace, g, weights, st);
  else if (tv && norm_out)
    dispatch_walk_tv<COPY_NONE, false>(layout, x, c, mask, planned, workspace, g, weights, st);
  else if (copy == COPY_X_TO_C)
    dispatch_walk<false, COPY_X_TO_C, false>(layout, x, c, mask, planned, workspace, g, st);
  else if (copy == COPY_C_TO_X && norm_out)
    dispatch_walk<true, COPY_C_TO_X, false>(layout, x, c, mask, planned, workspace, g, st);
  else if (copy == COPY_C_TO_X)
    dispatch_walk<false, COPY_C_TO_X, false>(layout, x, c, mask, planned, workspace, g, st);
  else
    dispatch_walk<true, COPY_NONE, false>(layout, x, c, mask, planned, workspace, g, st);
  if (norm_out && tv)
    launch_finish_tv((char*)workspace + kVarPartialOffset, g.n_wg, norm_out, st);
  else if (norm_out)
    launch_finish(layout->dtype, (char*)workspace + kVarPartialOffset, g.n_wg, norm_out, st);
  return launch_status();
}

}  // namespace scar

using namespace scar;

extern "C" size_t scar_var_workspace_bytes(uint64_t n_blocks) {
  return n_blocks > SCAR_MAX_BLOCKS ? 0 : var_workspace_bytes_for(n_blocks);
}

// Shared body of scar_var_block_scores and scar_var_tv_block_scores.
static int var_scores(bool tv, const scar_var_layout* layout, const void* x, const void* c,
                      const float* weights, void* scores, void* workspace, size_t workspace_bytes,
                      void* stream) {
  if (tv && layout && (layout->dtype == SCAR_I32 || layout->dtype == SCAR_F32_BF16C)) return SCAR_ERR_UNSUPPORTED;
  const uint64_t nb = var_blocks(layout);
  if (nb == UINT64_MAX) return SCAR_ERR_INVALID_ARG;
  if (nb == 0) return SCAR_OK;
  const int eb = host_elem_bytes(layout->dtype), ceb = host_c_elem_bytes(layout->dtype);
  if (!scores || !aligned(scores, layout->dtype == SCAR_I32 ? 8 : 4) || !aligned(weights, 4)) return SCAR_ERR_INVALID_ARG;
  if (layout->n_elems && (!x || !c || !aligned(x, eb) || !aligned(c, ceb))) return SCAR_ERR_INVALID_ARG;
  const int rc = check_var_workspace(workspace, workspace_bytes, nb);
  if (rc) return rc;
  hipStream_t st = (hipStream_t)stream;
  const VarGeometry g = var_geometry(layout->n_elems, kVarMaxGridCopy);
  if (tv) {
    if (layout->n_elems) dispatch_walk_tv<COPY_NONE, true>(layout, x, c, nullptr, false, workspace, g, weights, st);
    if (layout->dtype == SCAR_F32)
      launch_scores_finish<DT_F32_TV>(layout, workspace, g, scores, st, weights);
    else
      launch_scores_finish<DT_BF16_TV>(layout, workspace, g, scores, st, weights);
    return launch_status();
  }
  if (layout->n_elems) dispatch_walk<true, COPY_NONE, true>(layout, x, c, nullptr, false, workspace, g, st);
  switch (layout->dtype) {
    case SCAR_I32: launch_scores_finish<DT_I32>(layout, workspace, g, scores, st); break;
    default: launch_scores_finish<DT_F32>(layout, workspace, g, scores, st); break;
  }
  return launch_status();
}

extern "C" int scar_var_block_scores(const scar_var_layout* layout, const void* x, const void* c,
                                     void* scores, void* workspace, size_t workspace_bytes,
                                     void* stream) {
  return var_scores(false, layout, x, c, nullptr, scores, workspace, workspace_bytes, stream);
}

extern "C" int scar_var_tv_block_scores(const scar_var_layout* layout, const void* x, const void* c,
                                        const float* weights, float* scores, void* workspace,
                                        size_t workspace_bytes, void* stream) {
  return var_scores(true, layout, x, c, weights, scores, workspace, workspace_bytes, stream);
}

extern "C" int scar_var_tv_partial_recover(const scar_var_layout* layout, void* x, const void* c,
                                           const float* weights, const uint32_t* lost_idx, uint32_t n_lost,
                                           scar_norm* norm_out, void* workspace, size_t workspace_bytes,
                                           void* stream) {
  return var_rows(COPY_C_TO_X, layout, x, c, lost_idx, n_lost, false, norm_out, workspace, workspace_bytes,
                  stream, nullptr, nullptr, true, weights);
}

extern "C" int scar_var_tv_perturbation_norm(const scar_var_layout* layout, const void* x, const void* c,
                                             const float* weights, const uint32_t* idx, uint32_t n_idx,
                                             scar_norm* norm_out, void* workspace, size_t workspace_bytes,
                                             void* stream) {
  if (!norm_out) return SCAR_ERR_INVALID_ARG;
  return var_rows(COPY_NONE, layout, x, c, idx, n_idx, idx == nullptr, norm_out, workspace, workspace_bytes,
                  stream, nullptr, nullptr, true, weights);
}

extern "C" int scar_var_checkpoint_commit(const scar_var_layout* layout, const void* x, void* c,
                                          const uint32_t* idx, uint32_t n_idx, void* workspace,
                                          size_t workspace_bytes, void* stream) {
  return var_rows(COPY_X_TO_C, layout, x, c, idx, n_idx, false, nullptr, workspace, workspace_bytes,
                  stream);
}

extern "C" int scar_var_partial_recover(const scar_var_layout* layout, void* x, const void* c,
                                        const uint32_t* lost_idx, uint32_t n_lost, scar_norm* norm_out,
                                        void* workspace, size_t workspace_bytes, void* stream) {
  return var_rows(COPY_C_TO_X, layout, x, c, lost_idx, n_lost, false, norm_out, workspace,
                  workspace_bytes, stream);
}

extern "C" int scar_var_perturbation_norm(const scar_var_layout* layout, const void* x, const void* c,
                                          const uint32_t* idx, uint32_t n_idx, scar_norm* norm_out,
                                          void* workspace, size_t workspace_bytes, void* stream) {
  if (!norm_out) return SCAR_ERR_INVALID_ARG;
  return var_rows(COPY_NONE, layout, x, c, idx, n_idx, idx == nullptr, norm_out, workspace,
                  workspace_bytes, stream);
}

extern "C" int scar_var_checkpoint_commit_staged(const scar_var_layout* layout, const void* x, void* c,
                                                 const uint32_t* idx, uint32_t n_idx, void* staging,
                                                 uint64_t* staging_offsets, void* workspace,
                                                 size_t workspace_bytes, void* stream) {
  if (!staging_offsets || (n_idx && !staging)) return SCAR_ERR_INVALID_ARG;
  // with nothing listed the offsets are still written; any non-NULL side pointer will do
  return var_rows(COPY_X_TO_C, layout, x, c, idx, n_idx, false, nullptr, workspace, workspace_bytes, stream,
                  staging ? staging : (void*)staging_offsets, staging_offsets);
}

extern "C" int scar_var_partial_recover_rows(const scar_var_layout* layout, void* x, const void* rows,
                                             const uint64_t* row_offsets, const uint32_t* lost_idx,
                                             uint32_t n_lost, scar_norm* norm_out, void* workspace,
                                             size_t workspace_bytes, void* stream) {
  if (n_lost && (!rows || !row_offsets)) return SCAR_ERR_INVALID_ARG;
  if (n_lost == 0)  // nothing to take from the rows: the plain call writes the zero norm
    return var_rows(COPY_C_TO_X, layout, x, x, lost_idx, 0, false, norm_out, workspace, workspace_bytes, stream);
  return var_rows(COPY_C_TO_X, layout, x, x, lost_idx, n_lost, false, norm_out, workspace, workspace_bytes,
                  stream, const_cast<void*>(rows), const_cast<uint64_t*>(row_offsets));
}
