// Reduced-precision checkpoint (store type SCAR_F32_BF16C): the live parameters x are
// float32, the running checkpoint c is kept in bfloat16 (Example 2.1: a representation with
// a p-bit significand perturbs every element by less than 2^-(p-1) |y|).  The score scan
// then reads 6 bytes per parameter instead of 8.
//
//   scores / norm:  (x_j - widen(c_j))^2, c widened exactly (bfloat16 is the upper half of
//                   a float32)
//   commit:         c_j <- x_j rounded to nearest, ties to even
//   recovery:       x_j <- widen(c_j)
//
// The unit of work is 4 elements: a 16-byte vector of x against 8 bytes of c, so that
// consecutive lanes touch consecutive addresses in both streams.
#include "scar_device.hpp"
#include "scar_host.hpp"
#include "scar_mixed_device.hpp"

namespace scar {

// LISTED: only the blocks idx[0..n_idx) are scored (entries >= n_blocks are skipped); the other
// entries of scores stay as they are.
template <int G, bool LISTED>
__global__ __launch_bounds__(kWG) void k_mixed_scores(const float* __restrict__ x,
                                                      const uint16_t* __restrict__ c,
                                                      float* __restrict__ scores, uint64_t n_elems,
                                                      uint32_t block_len, uint32_t n_blocks,
                                                      const uint32_t* __restrict__ idx, uint32_t n_idx) {
  constexpr int GPW = (G == 256) ? 1 : kWG / G;
  const int lane = (G == 256) ? threadIdx.x : (threadIdx.x & (G - 1));
  const uint32_t grp = (G == 256) ? 0 : threadIdx.x / G;
  __shared__ double slots[kWG / kWave];
  const uint64_t n_items = LISTED ? n_idx : n_blocks;
  for (uint64_t i = (uint64_t)xcd_contiguous_block_id() * GPW + grp; i < n_items;
       i += (uint64_t)gridDim.x * GPW) {
    uint64_t b = i;
    if constexpr (LISTED) {
      b = idx[i];
      if (b >= n_blocks) continue;
    }
    const BlockSpan sp = block_span(b, n_elems, block_len, 1);  // byte_off = element offset
    const float* xb = x + sp.byte_off;
    const uint16_t* cb = c + sp.byte_off;
    double acc = mixed_distance<G>(xb, cb, sp.len, mixed_head(xb, cb, sp.len), lane);
    if constexpr (G == 256)
      acc = workgroup_sum(acc, slots);
    else
      acc = group_sum<G>(acc);
    if (lane == 0) scores[b] = (float)acc;
  }
}

// Many short rows of an aligned store, read as runs of whole rows (the reduced-precision twin
// of k_block_scores_flat): a workgroup loads a chunk of `chunk_rows` whole rows - at most
// kMixFlatUnits units per stream, every lane kMixU of them, fully coalesced - and leaves in LDS
// one partial sum per unit and, SPLIT (rows that are not whole units: a row then starts inside
// a unit and has leading and trailing elements of its own), one term per element as well.  The
// groups then add each row's values in the order in which mixed_distance adds them from memory
// (units, then the elements around them), so the scores are bit for bit those of
// k_mixed_scores, which still serves listed blocks and a short last block of the store.
// Chunks start on 16-byte boundaries of x (8-byte boundaries of c); the host sizes chunk_rows
// for that.
constexpr uint32_t kMixFlatUnits = kWG * kMixU;
constexpr uint32_t kMixFlatRowElems = 128;       // longest row of whole units taken (512 bytes of x)
constexpr uint32_t kMixFlatSplitRowElems = 256;  // longest row that is not
constexpr uint32_t kMixFlatMinRows = 4096;

template <int G, bool SPLIT>
__global__ __launch_bounds__(kWG) void k_mixed_scores_flat(const float* __restrict__ x,
                                                           const uint16_t* __restrict__ c,
                                                           float* __restrict__ scores, uint32_t block_len,
                                                           uint32_t n_rows, uint32_t chunk_rows,
                                                           uint32_t n_chunks) {
  constexpr int GPW = kWG / G;
  __shared__ float unit_sums[kMixFlatUnits];
  __shared__ __align__(16) float terms[SPLIT ? kMixFlatUnits * kMixUnit : 1];
  const int lane = threadIdx.x & (G - 1);
  const uint32_t grp = threadIdx.x / G;
  for (uint32_t chunk = xcd_contiguous_block_id(); chunk < n_chunks; chunk += gridDim.x) {
    const uint64_t row0 = (uint64_t)chunk * chunk_rows;
    const uint32_t rows = (uint32_t)(n_rows - row0 < chunk_rows ? n_rows - row0 : chunk_rows);
    const uint32_t n_el = rows * block_len;
    const uint32_t nunit = n_el / kMixUnit;  // whole units; only the last chunk can end inside one
    const float* xc = x + row0 * block_len;
    const uint16_t* cc = c + row0 * block_len;
    uint4 a[kMixU];
    uint2 b[kMixU];
#pragma unroll
    for (int u = 0; u < kMixU; ++u) {
      const uint32_t i = u * kWG + threadIdx.x;
      if (i < nunit) {
        a[u] = load_stream((const uint4*)xc + i);
        b[u] = load_stream2((const uint2*)cc + i);
      }
    }
#pragma unroll
    for (int u = 0; u < kMixU; ++u) {
      const uint32_t i = u * kWG + threadIdx.x;
      if (i >= nunit) continue;
      unit_sums[i] = sqdiff_unit(a[u], b[u]);
      if constexpr (SPLIT) {
        float4 t;  // the terms of the element-wise walk
        t.x = sq(__uint_as_float(a[u].x) - widen_lo(b[u].x));
        t.y = sq(__uint_as_float(a[u].y) - widen_hi(b[u].x));
        t.z = sq(__uint_as_float(a[u].z) - widen_lo(b[u].y));
        t.w = sq(__uint_as_float(a[u].w) - widen_hi(b[u].y));
        ((float4*)terms)[i] = t;
      }
    }
    if constexpr (SPLIT)  // the elements after the last whole unit (last chunk only)
      for (uint32_t j = nunit * kMixUnit + threadIdx.x; j < n_el; j += kWG) terms[j] = sq(xc[j] - widen_elem(cc, j));
    __syncthreads();
    for (uint32_t r = grp; r < rows; r += GPW) {
      double acc = 0;
      // the row's own split, as mixed_head makes it: chunks start on whole units
      const uint32_t e_lo = r * block_len;
      uint32_t head = SPLIT ? (uint32_t)(0 - e_lo) & (kMixUnit - 1) : 0;
      if (head > block_len) head = block_len;
      const uint32_t row_units = (block_len - head) / kMixUnit, tail0 = head + row_units * kMixUnit;
      const float* p = unit_sums + (e_lo + head) / kMixUnit;
      for (uint32_t u0 = 0; u0 < row_units; u0 += G * kMixU) {  // the order of mixed_distance
        float part = 0.f;
#pragma unroll
        for (int u = 0; u < kMixU; ++u) {
          const uint32_t i = u0 + u * G + lane;
          part += i < row_units ? p[i] : 0.f;
        }
        acc += (double)part;
      }
      if constexpr (SPLIT) {
        for (uint32_t e = lane; e < block_len - row_units * kMixUnit; e += G)
          acc += (double)terms[e_lo + (e < head ? e : tail0 + (e - head))];
      }
      acc = group_sum<G>(acc);
      if (lane == 0) scores[row0 + r] = (float)acc;
    }
    __syncthreads();  // the next chunk overwrites the sums and terms
  }
}

// Rows longer than kMixPieceElems elements (4 KiB of x) are handed out in pieces of that
// length, one per grid-y slice, like the rows of the other store types.
constexpr uint32_t kMixPieceElems = kPieceBytes / 4;

// Element range [first, first + len) of block b that piece `piece` covers; false if none.
__device__ __forceinline__ bool mixed_piece(uint32_t b, uint32_t piece, uint32_t pieces, uint32_t n_blocks,
                                            uint64_t n_elems, uint32_t block_len, uint64_t* elem_off,
                                            uint32_t* first, uint32_t* len) {
  if (b >= n_blocks) return false;
  const BlockSpan sp = block_span(b, n_elems, block_len, 1);  // byte_off = element offset
  *first = piece * kMixPieceElems;
  if (*first >= sp.len) return false;
  *len = sp.len - *first;
  if (pieces > 1 && *len > kMixPieceElems) *len = kMixPieceElems;
  *elem_off = sp.byte_off + *first;
  return true;
}

// c_b <- round(x_b) (and staging row i <- the same bfloat16 values) for b = idx[i].
// WHOLE: every row starts on a unit boundary of both streams and is a whole number of units
// (but for a short last block) - x 16-byte, c 8-byte aligned, block_len a multiple of 4 -
// so no row has leading elements and the split by addresses is skipped.
template <int G, bool WHOLE>
__global__ __launch_bounds__(kWG) void k_mixed_commit(const float* __restrict__ x, uint16_t* __restrict__ c,
                                                      const uint32_t* __restrict__ idx, uint32_t n_idx,
                                                      uint16_t* __restrict__ staging, uint64_t n_elems,
                                                      uint32_t block_len, uint32_t n_blocks, uint32_t pieces) {
  constexpr int GPW = (G == 256) ? 1 : kWG / G;
  const int lane = (G == 256) ? threadIdx.x : (threadIdx.x & (G - 1));
  const uint32_t grp = (G == 256) ? 0 : threadIdx.x / G;
  const GridSlot slot = row_grid_slot(((uint64_t)n_idx + GPW - 1) / GPW);
  for (uint32_t piece = slot.y; piece < pieces; piece += gridDim.y) {
    for (uint64_t i = (uint64_t)slot.x * GPW + grp; i < n_idx;
         i += (uint64_t)gridDim.x * GPW) {
      uint64_t off;
      uint32_t first, len;
      if (!mixed_piece(idx[i], piece, pieces, n_blocks, n_elems, block_len, &off, &first, &len)) continue;
      const float* xb = x + off;
      uint16_t* cb = c + off;
      uint16_t* sb = staging ? staging + i * (uint64_t)block_len + first : nullptr;
      const uint32_t head = WHOLE ? 0 : mixed_head(xb, cb, len);
      // the staging row takes whole units too if it has the phase of c's row
      const bool vec_staging = sb && (((uintptr_t)sb ^ (uintptr_t)cb) & 7) == 0;
      const uint32_t nunit = (len - head) / kMixUnit, tail0 = head + nunit * kMixUnit;
      // the few elements around the whole units are asked for together with the first units when
      // the group has a lane for each of them; a row walked element by element loops instead
      const bool ends_in_lanes = !WHOLE && G >= kMixUnit && head < (uint32_t)kMixUnit;
      const bool has_head = ends_in_lanes && (uint32_t)lane < head, has_tail = ends_in_lanes && tail0 + lane < len;
      uint32_t hx = 0, tx = 0;
      if (has_head) hx = __float_as_uint(xb[lane]);
      if (has_tail) tx = __float_as_uint(xb[tail0 + lane]);
      auto element = [&](uint32_t j) {
        const uint16_t r = (uint16_t)round_bf16(__float_as_uint(xb[j]));
        cb[j] = r;
        if (sb) sb[j] = r;
      };
      if (!ends_in_lanes)
        for (uint32_t j = lane; j < head; j += G) element(j);
      for (uint32_t u = lane; u < nunit; u += G) {
        const uint2 r = round_unit(load_stream((const uint4*)(xb + head) + u));
        store_stream2((uint2*)(cb + head) + u, r);
        if (sb && vec_staging) store_stream2((uint2*)(sb + head) + u, r);
      }
      if (has_head) {
        const uint16_t r = (uint16_t)round_bf16(hx);
        cb[lane] = r;
        if (sb) sb[lane] = r;
      }
      if (has_tail) {
        const uint16_t r = (uint16_t)round_bf16(tx);
        cb[tail0 + lane] = r;
        if (sb) sb[tail0 + lane] = r;
      }
      if (!ends_in_lanes)
        for (uint32_t j = tail0 + lane; j < len; j += G) element(j);
      if (sb && !vec_staging)
        for (uint32_t j = head + lane; j < tail0; j += G) sb[j] = (uint16_t)round_bf16(__float_as_uint(xb[j]));
    }
  }
}

// Recovery and/or norm over the blocks idx[0..n_idx) (idx == NULL: blocks 0..n_idx), with T
// threads per workgroup (1,024 for long index lists, so that no group takes a second entry).
template <int G, int T, bool STORE, bool NORM, bool WHOLE>
__global__ __launch_bounds__(T) void k_mixed_recover(float* __restrict__ x, const uint16_t* __restrict__ c,
                                                     const uint32_t* __restrict__ idx, uint32_t n_idx,
                                                     uint64_t n_elems, uint32_t block_len,
                                                     uint32_t n_blocks, uint32_t pieces, bool packed,
                                                     double* __restrict__ partial) {
  constexpr int GPW = T / G;
  const int lane = threadIdx.x & (G - 1);
  const uint32_t grp = threadIdx.x / G;
  __shared__ double slots[T / kWave];
  double acc = 0;
  const GridSlot slot = row_grid_slot(((uint64_t)n_idx + GPW - 1) / GPW);
  for (uint32_t piece = slot.y; piece < pieces; piece += gridDim.y) {
    for (uint64_t i = (uint64_t)slot.x * GPW + grp; i < n_idx;
         i += (uint64_t)gridDim.x * GPW) {
      uint64_t off;
      uint32_t first, len;
      if (!mixed_piece(idx ? idx[i] : (uint32_t)i, piece, pieces, n_blocks, n_elems, block_len, &off, &first,
                       &len))
        continue;
      float* xb = x + off;
      const uint16_t* cb = packed ? c + i * (uint64_t)block_len + first : c + off;
      const uint32_t head = WHOLE ? 0 : mixed_head(xb, cb, len);
      const uint32_t nunit = (len - head) / kMixUnit, tail0 = head + nunit * kMixUnit;
      const bool ends_in_lanes = !WHOLE && G >= kMixUnit && head < (uint32_t)kMixUnit;  // as in k_mixed_commit
      const bool has_head = ends_in_lanes && (uint32_t)lane < head, has_tail = ends_in_lanes && tail0 + lane < len;
      float hc = 0, hx = 0, tc = 0, tx = 0;
      if (has_head) {
        hc = widen_elem(cb, lane);
        if (NORM) hx = xb[lane];
      }
      if (has_tail) {
        tc = widen_elem(cb, tail0 + lane);
        if (NORM) tx = xb[tail0 + lane];
      }
      auto element = [&](uint32_t j) {
        const float w = widen_elem(cb, j);
        if (NORM) acc += (double)sq(xb[j] - w);
        if (STORE) xb[j] = w;
      };
      if (!ends_in_lanes)
        for (uint32_t j = lane; j < head; j += G) element(j);
      if (NORM && has_head) acc += (double)sq(hx - hc);
      for (uint32_t u = lane; u < nunit; u += G) {
        const uint2 cv = load_stream2((const uint2*)(cb + head) + u);
        if (NORM) acc += (double)sqdiff_unit(load_stream((const uint4*)(xb + head) + u), cv);
        if (STORE) store_stream((uint4*)(xb + head) + u, widen_unit(cv));
      }
      if (NORM && has_tail) acc += (double)sq(tx - tc);
      if (STORE) {
        if (has_head) xb[lane] = hc;
        if (has_tail) xb[tail0 + lane] = tc;
      }
      if (!ends_in_lanes)
        for (uint32_t j = tail0 + lane; j < len; j += G) element(j);
    }
  }
  if (NORM) {
    acc = workgroup_sum<T>(acc, slots);
    if (threadIdx.x == 0) partial[blockIdx.y * gridDim.x + blockIdx.x] = acc;
  }
}

#define SCAR_FOR_GROUP(g, CALL)  \
  switch (g) {                   \
    case 1: CALL(1); break;      \
    case 2: CALL(2); break;      \
    case 4: CALL(4); break;      \
    case 8: CALL(8); break;      \
    case 16: CALL(16); break;    \
    case 32: CALL(32); break;    \
    case 64: CALL(64); break;    \
    case 128: CALL(128); break;  \
    default: CALL(256); break;   \
  }

// x and c start at the same phase (mixed_head), so the rows of the store are walked in whole
// units: what the launches are sized for.  The kernels decide row by row.
static bool mixed_vec(const void* x, const void* c) {
  return ((reinterpret_cast<uintptr_t>(x) >> 2) & (kMixUnit - 1)) == ((reinterpret_cast<uintptr_t>(c) >> 1) & (kMixUnit - 1));
}

// Rows of whole units: packed rows (staging, rows read back) then share the phase of the store's rows.
static bool unit_rows(const scar_layout* l) { return l->block_len % kMixUnit == 0; }

// Every row starts on a unit boundary of both streams and is made of whole units.
static bool mixed_whole(const scar_layout* l, const void* x, const void* c) {
  return aligned(x, 16) && aligned(c, 8) && unit_rows(l);
}

// Lanes per row of the copy kernels: one per unit, and at least 4 for rows that are not whole
// units, so that the elements around the units each find a lane.
static int mixed_copy_group(const scar_layout* l, bool vec) {
  if (!vec) return pick_group_units(l->block_len, 1, true);
  const int g = pick_group_units((l->block_len + kMixUnit - 1) / kMixUnit, 1, true);
  return (!unit_rows(l) && g < kMixUnit) ? kMixUnit : g;
}

// Pieces per row for the copy kernels (1 unless the rows are walked in units and exceed a piece).
static uint32_t mixed_pieces(const scar_layout* l, bool vec) {
  return (vec && l->block_len > kMixPieceElems) ? (l->block_len + kMixPieceElems - 1) / kMixPieceElems : 1;
}

int mixed_block_scores(const scar_layout* l, uint32_t n_blocks, const void* x, const void* c,
                       const uint32_t* idx, uint32_t n_idx, void* scores, hipStream_t st) {
  if (!x || !c || !scores || !aligned(x, 4) || !aligned(c, 2) || !aligned(scores, 4))
    return SCAR_ERR_INVALID_ARG;
  int giant_status = SCAR_OK;  // a few very long blocks: cut into pieces, many workgroups per block
  if (mixed_giant_scores(l, n_blocks, x, c, idx, n_idx, scores, st, &giant_status)) return giant_status;
  const bool vec = mixed_vec(x, c);
  // loads in flight: one 16-byte step of x and 8 bytes of c per unit (element-wise: 4 + 2)
  const uint64_t units = vec ? (l->block_len + kMixUnit - 1) / kMixUnit : l->block_len;
  const int g = pick_group_units(units, vec ? kMixU : 4, false);
  // many short rows of an aligned store: read as runs of whole rows, added up in the order of
  // the group walk with the same g
  const bool split = !unit_rows(l);
  if (!idx && aligned(x, 16) && aligned(c, 8) && n_blocks >= kMixFlatMinRows && g <= 64 &&
      l->block_len <= (split ? kMixFlatSplitRowElems : kMixFlatRowElems) &&
      run_chunk_rows((uint64_t)l->block_len * 4, kMixFlatUnits) > 0) {
    const uint32_t n_rows = (uint32_t)(l->n_elems / l->block_len);
    const uint32_t chunk_rows = run_chunk_rows((uint64_t)l->block_len * 4, kMixFlatUnits);  // sized by the rows of x
    const uint32_t n_chunks = (n_rows + chunk_rows - 1) / chunk_rows;
    const uint32_t grid = xcd_grid(n_chunks, kScoreGridCap);
    // four workgroups per compute unit: 40 KiB of LDS each, part of it unused
    const size_t used = (split ? kMixFlatUnits * (kMixUnit + 1) : kMixFlatUnits) * sizeof(float) + 256;
    const size_t lds = 40 * 1024 - used;
#define FLAT(G)                                                                                        \
  case G:                                                                                              \
    if (split)                                                                                         \
      launch((k_mixed_scores_flat<G, true>), dim3(grid), dim3(kWG), lds, st,               \
                         (const float*)x, (const uint16_t*)c, (float*)scores, l->block_len, n_rows,    \
                         chunk_rows, n_chunks);                                                        \
    else                                                                                               \
      launch((k_mixed_scores_flat<G, false>), dim3(grid), dim3(kWG), lds, st,              \
                         (const float*)x, (const uint16_t*)c, (float*)scores, l->block_len, n_rows,    \
                         chunk_rows, n_chunks);                                                        \
    break;
    switch (g) {
      FLAT(1) FLAT(2) FLAT(4) FLAT(8) FLAT(16) FLAT(32) FLAT(64)
    }
#undef FLAT
    const uint64_t done = (uint64_t)n_rows * l->block_len;
    if (done == l->n_elems) return launch_status();
    // a short last block: a store of one block for the group walk below
    const scar_layout last = {l->dtype, l->block_len, l->n_elems - done};
    return mixed_block_scores(&last, 1, (const float*)x + done, (const uint16_t*)c + done, nullptr, 0,
                              (float*)scores + n_rows, st);
  }
#define CALL(G)                                                                                      \
  {                                                                                                  \
    constexpr int GPW = (G == 256) ? 1 : kWG / G;                                                    \
    const uint64_t need = ((uint64_t)(idx ? n_idx : n_blocks) + GPW - 1) / GPW;                      \
    const uint32_t grid = xcd_grid(need, kScoreGridCap);                                             \
    const uint64_t group_units = units < (uint64_t)G * kMixU ? units : (uint64_t)G * kMixU;          \
    const size_t lds = stream_lds_bytes(need, (vec ? 24 : 6) * group_units * GPW);                   \
    if (idx)                                                                                         \
      launch((k_mixed_scores<G, true>), dim3(grid), dim3(kWG), lds, st, (const float*)x, \
                         (const uint16_t*)c, (float*)scores, l->n_elems, l->block_len, n_blocks,     \
                         idx, n_idx);                                                                \
    else                                                                                             \
      launch((k_mixed_scores<G, false>), dim3(grid), dim3(kWG), lds, st,                 \
                         (const float*)x, (const uint16_t*)c, (float*)scores, l->n_elems,            \
                         l->block_len, n_blocks, idx, n_idx);                                        \
  }
  switch (g) {  // the score kernel reduces inside a wavefront or a whole workgroup
    case 1: CALL(1) break;
    case 2: CALL(2) break;
    case 4: CALL(4) break;
    case 8: CALL(8) break;
    case 16: CALL(16) break;
    case 32: CALL(32) break;
    case 64: CALL(64) break;
    default: CALL(256) break;
  }
#undef CALL
  return launch_status();
}

int mixed_commit(const scar_layout* l, uint32_t n_blocks, const void* x, void* c, const uint32_t* idx,
                 uint32_t n_idx, void* staging, hipStream_t st) {
  if (!x || !c || !idx || !aligned(x, 4) || !aligned(c, 2) || !aligned(idx, 4) ||
      (staging && !aligned(staging, 2)))
    return SCAR_ERR_INVALID_ARG;
  const bool vec = mixed_vec(x, c);
  const bool whole = mixed_whole(l, x, c);
  const uint32_t pieces = mixed_pieces(l, vec);
  const int g = pieces > 1 ? 256 : mixed_copy_group(l, vec);
#define CALL(G)                                                                                     \
  {                                                                                                 \
    constexpr int GPW = (G == 256) ? 1 : kWG / G;                                                   \
    const RowGrid rg = row_grid(((uint64_t)n_idx + GPW - 1) / GPW, pieces, kCopyGridCap);           \
    if (whole)                                                                                      \
      launch((k_mixed_commit<G, true>), dim3(rg.x, rg.y), dim3(kWG), 0, st, (const float*)x, (uint16_t*)c, idx, \
             n_idx, (uint16_t*)staging, l->n_elems, l->block_len, n_blocks, pieces);                \
    else                                                                                            \
      launch((k_mixed_commit<G, false>), dim3(rg.x, rg.y), dim3(kWG), 0, st, (const float*)x, (uint16_t*)c, idx, \
             n_idx, (uint16_t*)staging, l->n_elems, l->block_len, n_blocks, pieces);                \
  }
  SCAR_FOR_GROUP(g, CALL)
#undef CALL
  return launch_status();
}

template <bool STORE, bool NORM, bool WHOLE>
static uint32_t launch_mixed_recover(int g, const scar_layout* l, uint32_t n_blocks, void* x,
                                     const void* c, const uint32_t* idx, uint32_t n_idx, uint32_t pieces,
                                     bool packed, void* partial, hipStream_t st) {
  uint32_t grid = 0, grid_y = 1;
  constexpr int kWide = 1024;
#define LAUNCH(G, T)                                                                                  \
  {                                                                                                   \
    const RowGrid rg = row_grid(((uint64_t)n_idx + (T / G) - 1) / (T / G), pieces, kMaxNormGrid);     \
    grid = rg.x, grid_y = rg.y;                                                                       \
    launch((k_mixed_recover<G, T, STORE, NORM, WHOLE>), dim3(grid, grid_y), dim3(T), 0, st, \
                       (float*)x, (const uint16_t*)c, idx, n_idx, l->n_elems, l->block_len, n_blocks, \
                       pieces, packed, (double*)partial);                                             \
  }
#define CALL(G)                                                       \
  if (n_idx >= 64 && ((uint64_t)n_idx * pieces * G + kWG - 1) / kWG >= 8192) \
    LAUNCH(G, kWide)                                                  \
  else                                                                \
    LAUNCH(G, kWG)
  SCAR_FOR_GROUP(g, CALL)
#undef CALL
#undef LAUNCH
  return grid * grid_y;
}

// The norm over the whole store with nothing stored: one flat reduction over units of 4
// elements, kMixU of them per lane in flight, each unit's float32 sum folded into float64 on
// its own as the row walk does it.  Needs x 16-byte and c 8-byte aligned; the elements after
// the last whole unit go to the first workgroup.
__global__ __launch_bounds__(kWG) void k_mixed_norm_all(const float* __restrict__ x,
                                                        const uint16_t* __restrict__ c, uint64_t n_elems,
                                                        double* __restrict__ partial) {
  __shared__ double slots[kWG / kWave];
  const uint64_t nunit = n_elems / kMixUnit;
  double acc = 0;
  for (uint64_t u0 = (uint64_t)xcd_contiguous_block_id() * (kWG * kMixU); u0 < nunit;
       u0 += (uint64_t)gridDim.x * (kWG * kMixU)) {
    uint4 a[kMixU];
    uint2 b[kMixU];
#pragma unroll
    for (int u = 0; u < kMixU; ++u) {
      const uint64_t i = u0 + (uint64_t)u * kWG + threadIdx.x;
      if (i < nunit) {
        a[u] = load_stream((const uint4*)x + i);
        b[u] = load_stream2((const uint2*)c + i);
      } else {
        a[u] = make_uint4(0, 0, 0, 0);
        b[u] = make_uint2(0, 0);
      }
    }
#pragma unroll
    for (int u = 0; u < kMixU; ++u) acc += (double)sqdiff_unit(a[u], b[u]);
  }
  if (blockIdx.x == 0)
    for (uint64_t j = nunit * kMixUnit + threadIdx.x; j < n_elems; j += kWG)
      acc += (double)sq(x[j] - widen_elem(c, j));
  acc = workgroup_sum(acc, slots);
  if (threadIdx.x == 0) partial[blockIdx.x] = acc;
}

int mixed_recover_or_norm(bool store, bool packed, const scar_layout* l, uint32_t n_blocks, void* x,
                          const void* c,
                          const uint32_t* idx, uint32_t n_idx, scar_norm* norm_out, void* partial,
                          hipStream_t st) {
  if (!aligned(x, 4) || !aligned(c, 2)) return SCAR_ERR_INVALID_ARG;
  const bool vec = mixed_vec(x, c) && (!packed || unit_rows(l));  // c = packed rows: their own phase
  const uint32_t pieces = mixed_pieces(l, vec);
  const int g = pieces > 1 ? 256 : mixed_copy_group(l, vec);
  uint32_t n_partial = 0;
  if (!store && norm_out && !idx && !packed && aligned(x, 16) && aligned(c, 8)) {  // the whole store
    const uint64_t chunks = (l->n_elems / kMixUnit + kWG * kMixU - 1) / (kWG * kMixU);
    const uint32_t grid = xcd_grid(chunks ? chunks : 1, kMaxNormGrid);
    launch(k_mixed_norm_all, dim3(grid), dim3(kWG), stream_lds_bytes(grid, 24 * kWG * kMixU), st,
                       (const float*)x, (const uint16_t*)c, l->n_elems, (double*)partial);
    launch_finish(l->dtype, partial, grid, norm_out, st);
    return launch_status();
  }
  const bool whole = mixed_whole(l, x, c);  // c = packed rows included: rows of whole units keep its phase
#define RUN(STORE, NORM, PARTIAL)                                                                              \
  (whole ? launch_mixed_recover<STORE, NORM, true>(g, l, n_blocks, x, c, idx, n_idx, pieces, packed, PARTIAL, st) \
         : launch_mixed_recover<STORE, NORM, false>(g, l, n_blocks, x, c, idx, n_idx, pieces, packed, PARTIAL, st))
  if (store && norm_out)
    n_partial = RUN(true, true, partial);
  else if (store)
    RUN(true, false, nullptr);
  else
    n_partial = RUN(false, true, partial);
#undef RUN
  if (norm_out) launch_finish(l->dtype, partial, n_partial, norm_out, st);
  return launch_status();
}

}  // namespace scar
