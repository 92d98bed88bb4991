// scar_block_scores: distance of every block of x from the running checkpoint c
// (checkpoint step 1 of Section 4.3).
//
// The kernel is a pure two-stream read: 2 * n_elems * element-size bytes in, one score
// per block out.  G lanes walk one block with 16-byte loads from x and from c issued
// back to back (kUnroll of each before the first use), the per-lane sums are combined
// with wavefront shuffles (G <= 64) or shuffles plus one LDS step (G = 256).  Loads are
// non-temporal and each XCD walks one contiguous eighth of the store.
#include <mutex>

#include "scar_device.hpp"
#include "scar_host.hpp"
#include "scar_mixed_device.hpp"

namespace scar {

// LISTED: only the blocks idx[0..n_idx) are scored (entries >= n_blocks are skipped) and the
// other entries of scores stay as they are; otherwise every block is.
template <int DT, int G, bool VEC, bool LISTED>
__global__ __launch_bounds__(kWG) void k_block_scores(const char* __restrict__ x,
                                                      const char* __restrict__ c,
                                                      void* __restrict__ scores, uint64_t n_elems,
                                                      uint32_t block_len, uint32_t n_blocks,
                                                      const float* __restrict__ weights,
                                                      const uint32_t* __restrict__ idx, uint32_t n_idx) {
  constexpr int GPW = (G == 256) ? 1 : kWG / G;  // groups (= blocks in flight) per workgroup
  using acc_t = typename Acc<DT>::type;
  const int lane = (G == 256) ? threadIdx.x : (threadIdx.x & (G - 1));
  const uint32_t grp = (G == 256) ? 0 : threadIdx.x / G;
  __shared__ acc_t slots[kWG / kWave];

  const uint64_t n_items = LISTED ? n_idx : n_blocks;
  for (uint64_t i = (uint64_t)xcd_contiguous_block_id() * GPW + grp; i < n_items;
       i += (uint64_t)gridDim.x * GPW) {
    uint64_t b = i;
    if constexpr (LISTED) {
      b = idx[i];
      if (b >= n_blocks) continue;
    }
    const BlockSpan sp = block_span(b, n_elems, block_len, elem_bytes(DT));
    float w = 1.f;  // asked for before the walk, so that it has arrived when the walk is done
    if constexpr (is_tv(DT))
      if (weights && lane == 0) w = weights[b];
    acc_t acc = block_distance<DT, G, VEC>(x + sp.byte_off, c + sp.byte_off, sp.len, lane);
    if constexpr (G == 256)
      acc = workgroup_sum(acc, slots);
    else
      acc = group_sum<G>(acc);
    if (lane == 0) {
      if constexpr (DT == DT_I32)
        ((long long*)scores)[b] = (long long)acc;
      else if constexpr (is_tv(DT))  // w_b * 1/2 * sum |x - c|
        ((float*)scores)[b] = (float)(0.5 * acc * (double)w);
      else
        ((float*)scores)[b] = (float)acc;
    }
  }
}

// Rows shorter than 16 bytes (selection per scalar or per pair, block_len = 1, 2 or 4): a group
// per row would leave a lane with 4 or 8 bytes to fetch.  Here a lane takes a whole 16-byte
// step of x and of c - RPV = 16 / row bytes rows - and writes their RPV scores; the terms are
// added as the element-wise walk adds them, so the values are the same bit for bit.
// Needs 16-byte aligned bases; the elements after the last whole step (fewer than one step)
// are scored by the first lanes of the first workgroup.
template <int DT, int EPR>
__global__ __launch_bounds__(kWG) void k_block_scores_tiny(const char* __restrict__ x,
                                                           const char* __restrict__ c,
                                                           void* __restrict__ scores, uint64_t n_elems) {
  constexpr int E = elem_bytes(DT);
  constexpr int EPV = 16 / E;
  constexpr int RPV = EPV / EPR;
  using acc_t = typename Acc<DT>::type;
  const uint64_t nvec = n_elems / EPV;
  auto put = [&](uint64_t row, acc_t acc) {
    if constexpr (DT == DT_I32)
      ((long long*)scores)[row] = (long long)acc;
    else
      ((float*)scores)[row] = (float)acc;
  };
  for (uint64_t v0 = (uint64_t)xcd_contiguous_block_id() * kWG * kUnroll; v0 < nvec;
       v0 += (uint64_t)gridDim.x * kWG * kUnroll) {
    uint4 a[kUnroll], b[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const uint64_t v = v0 + (uint64_t)u * kWG + threadIdx.x;
      if (v < nvec) {
        a[u] = load_stream((const uint4*)x + v);
        b[u] = load_stream((const uint4*)c + v);
      }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const uint64_t v = v0 + (uint64_t)u * kWG + threadIdx.x;
      if (v >= nvec) continue;
#pragma unroll
      for (int r = 0; r < RPV; ++r) {
        acc_t acc = 0;
#pragma unroll
        for (int e = 0; e < EPR; ++e)  // element r * EPR + e of the 16 bytes held in registers
          accumulate_elem<DT>(acc, (const char*)&a[u], (const char*)&b[u], (uint64_t)(r * EPR + e));
        put(v * RPV + r, acc);
      }
    }
  }
  // what is left after the last whole step: fewer than EPV elements, i.e. fewer than RPV + 1 rows
  if (blockIdx.x == 0) {
    const uint64_t first_row = nvec * RPV;
    const uint64_t row = first_row + threadIdx.x;
    const uint64_t lo = row * EPR;
    if (threadIdx.x <= RPV && lo < n_elems) {
      const uint64_t hi = lo + EPR < n_elems ? lo + EPR : n_elems;
      acc_t acc = 0;
      for (uint64_t j = lo; j < hi; ++j) accumulate_elem<DT>(acc, x, c, j);
      put(row, acc);
    }
  }
}

template <int DT>
static bool launch_scores_tiny(const scar_layout* l, const void* x, const void* c, void* scores,
                               hipStream_t st) {
  constexpr int E = elem_bytes(DT);
  const uint64_t nvec = l->n_elems / (16 / E);
  const uint64_t need = (nvec + (uint64_t)kWG * kUnroll - 1) / ((uint64_t)kWG * kUnroll);
  const uint32_t grid = xcd_grid(need ? need : 1, kScoreGridCap);
#define SCAR_TINY(EPR)                                                                                  \
  launch((k_block_scores_tiny<DT, EPR>), dim3(grid), dim3(kWG), 0, st, (const char*)x,     \
                     (const char*)c, scores, l->n_elems)
  switch (l->block_len * E) {
    case 2: if constexpr (E == 2) { SCAR_TINY(1); return true; } return false;
    case 4: SCAR_TINY(4 / E); return true;
    case 8: SCAR_TINY(8 / E); return true;
    default: return false;
  }
#undef SCAR_TINY
}

template <int DT, int G>
static void launch_scores(const scar_layout* l, const void* x, const void* c, void* scores,
                          uint32_t n_blocks, bool vec, const float* weights, const uint32_t* idx,
                          uint32_t n_idx, hipStream_t st) {
  constexpr int GPW = (G == 256) ? 1 : kWG / G;
  const uint64_t need = ((uint64_t)(idx ? n_idx : n_blocks) + GPW - 1) / GPW;
  const uint32_t grid = xcd_grid(need, kScoreGridCap);
  // loads a workgroup keeps in flight: up to kUnroll 16-byte steps per lane and stream
  const uint64_t row_vecs = ((uint64_t)l->block_len * elem_bytes(DT) + 15) / 16;
  const uint64_t group_vecs = row_vecs < (uint64_t)G * kUnroll ? row_vecs : (uint64_t)G * kUnroll;
  const size_t lds = stream_lds_bytes(need, 2 * 16 * group_vecs * GPW);
#define SCAR_LAUNCH(VEC, LISTED)                                                                            \
  launch((k_block_scores<DT, G, VEC, LISTED>), dim3(grid), dim3(kWG), lds, st, (const char*)x, \
                     (const char*)c, scores, l->n_elems, l->block_len, n_blocks, weights, idx, n_idx)
  if (idx) {
    if (vec)
      SCAR_LAUNCH(true, true);
    else
      SCAR_LAUNCH(false, true);
  } else {
    if (vec)
      SCAR_LAUNCH(true, false);
    else
      SCAR_LAUNCH(false, false);
  }
#undef SCAR_LAUNCH
}

// Many short rows of a 16-byte aligned store, read as runs of whole rows.  A group per row
// reads such rows in pieces that start and end inside cache lines, leaves lanes idle (25 steps
// over 16 lanes) and, when a row is not a whole number of 16-byte steps, walks its ends element
// by element from memory.  Here a workgroup reads a *chunk* of `chunk_rows` whole rows as one
// contiguous run of at most kFlatVecs 16-byte steps per stream, every lane loading kUnroll of
// them fully coalesced, and leaves in LDS one partial sum per step and - SPLIT, for rows that
// are not whole steps - one term per element.  The groups then add each row's partial sums and
// terms in exactly the order in which block_distance adds them from memory (leading elements,
// steps, trailing elements; same lane -> step mapping, same float and float64 stages, same
// shuffles), so the scores are bit for bit those of k_block_scores - which still serves listed
// blocks.  Only whole rows are handled (n_rows of them); a short last block of the store is
// left to k_block_scores.  Chunks start on 16-byte boundaries (the host sizes chunk_rows for
// that), on 128-byte lines when the rows allow it.
constexpr uint32_t kFlatVecs = kWG * kUnroll;
constexpr uint32_t kFlatRowBytes = 512;        // longest row that is a whole number of steps
constexpr uint32_t kFlatSplitRowBytes = 4096 + 15;  // longest row that is not
constexpr uint32_t kFlatMinRows = 4096;        // below this a launch is all the time there is

template <int DT>
struct StepSum {
  using type = float;  // sum of the terms of one 16-byte step
};
template <>
struct StepSum<DT_I32> {
  using type = unsigned long long;
};
template <int DT>
struct ElemTerm {
  using type = float;  // term of a single element
};
template <>
struct ElemTerm<DT_I32> {
  using type = uint32_t;
};

// Distance term of element e (a compile-time constant) of a 16-byte step, as accumulate_elem
// computes it from memory.
template <int DT>
__device__ __forceinline__ typename ElemTerm<DT>::type elem_term(const uint4& a, const uint4& b, int e) {
  const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
  if constexpr (DT == DT_I32) {
    return absdiff_i32(aw[e], bw[e]);
  } else if constexpr (DT == DT_F32 || DT == DT_F32_TV) {
    const float d = __uint_as_float(aw[e]) - __uint_as_float(bw[e]);
    return DT == DT_F32 ? sq(d) : __builtin_fabsf(d);
  } else {
    const uint32_t ua = (e & 1) ? (aw[e / 2] & 0xffff0000u) : (aw[e / 2] << 16);
    const uint32_t ub = (e & 1) ? (bw[e / 2] & 0xffff0000u) : (bw[e / 2] << 16);
    const float d = __uint_as_float(ua) - __uint_as_float(ub);
    return DT == DT_BF16 ? sq(d) : __builtin_fabsf(d);
  }
}

template <int DT, int G, bool SPLIT>
__global__ __launch_bounds__(kWG) void k_block_scores_flat(const char* __restrict__ x,
                                                           const char* __restrict__ c,
                                                           void* __restrict__ scores, uint32_t block_len,
                                                           uint32_t n_rows, uint32_t chunk_rows,
                                                           uint32_t n_chunks,
                                                           const float* __restrict__ weights) {
  constexpr int E = elem_bytes(DT);
  constexpr int EPV = 16 / E;
  constexpr int GPW = kWG / G;
  using acc_t = typename Acc<DT>::type;
  using step_t = typename StepSum<DT>::type;
  using term_t = typename ElemTerm<DT>::type;
  __shared__ step_t steps[kFlatVecs];
  __shared__ __align__(16) term_t terms[SPLIT ? kFlatVecs * EPV : 1];
  __shared__ float row_weight[is_tv(DT) ? kFlatVecs / 2 : 1];  // rows are 32 bytes or more
  const int lane = threadIdx.x & (G - 1);
  const uint32_t grp = threadIdx.x / G;

  for (uint32_t chunk = xcd_contiguous_block_id(); chunk < n_chunks; chunk += gridDim.x) {
    const uint64_t row0 = (uint64_t)chunk * chunk_rows;
    const uint32_t rows = (uint32_t)(n_rows - row0 < chunk_rows ? n_rows - row0 : chunk_rows);
    const uint32_t n_el = rows * block_len;
    const uint32_t nvec = n_el / EPV;  // whole steps; only the last chunk can end inside one
    const char* xc = x + row0 * block_len * E;
    const char* cc = c + row0 * block_len * E;
    const uint4* xv = (const uint4*)xc;
    const uint4* cv = (const uint4*)cc;
    float w[2] = {1.f, 1.f};  // the rows' weights travel with the rows
    if constexpr (is_tv(DT)) {
      if (weights) {
#pragma unroll
        for (int u = 0; u < 2; ++u)
          if (u * kWG + threadIdx.x < rows) w[u] = weights[row0 + u * kWG + threadIdx.x];
      }
    }
    uint4 a[kUnroll], b[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const uint32_t v = u * kWG + threadIdx.x;
      if (v < nvec) {
        a[u] = load_stream(xv + v);
        b[u] = load_stream(cv + v);
      }
    }
    if constexpr (is_tv(DT)) {
#pragma unroll
      for (int u = 0; u < 2; ++u)
        if (u * kWG + threadIdx.x < rows) row_weight[u * kWG + threadIdx.x] = w[u];
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const uint32_t v = u * kWG + threadIdx.x;
      if (v >= nvec) continue;
      if constexpr (DT == DT_I32) steps[v] = absdiff_i32x4(a[u], b[u]);
      if constexpr (DT == DT_F32) steps[v] = sqdiff_f32(a[u], b[u]);
      if constexpr (DT == DT_BF16) steps[v] = sqdiff_bf16(a[u], b[u]);
      if constexpr (DT == DT_F32_TV) steps[v] = absdiff_f32(a[u], b[u]);
      if constexpr (DT == DT_BF16_TV) steps[v] = absdiff_bf16(a[u], b[u]);
      if constexpr (SPLIT) {
#pragma unroll
        for (int e = 0; e < EPV; ++e) terms[v * EPV + e] = elem_term<DT>(a[u], b[u], e);
      }
    }
    if constexpr (SPLIT) {  // the elements after the last whole step (last chunk only)
      for (uint32_t j = nvec * EPV + threadIdx.x; j < n_el; j += kWG) {
        acc_t t = 0;
        accumulate_elem<DT>(t, xc, cc, j);
        terms[j] = (term_t)t;
      }
    }
    __syncthreads();
    for (uint32_t r = grp; r < rows; r += GPW) {
      acc_t acc = 0;
      uint32_t head = 0, row_vecs = block_len / EPV, first_vec = r * row_vecs;
      const uint32_t e_lo = r * block_len;
      if constexpr (SPLIT) {  // the row's own split, as row_split makes it
        head = (EPV - (e_lo & (EPV - 1))) & (EPV - 1);
        if (head > block_len) head = block_len;
        row_vecs = (block_len - head) / EPV;
        first_vec = (e_lo + head) / EPV;
        for (uint32_t j = lane; j < head; j += G) acc += (acc_t)terms[e_lo + j];
      }
      const step_t* p = steps + first_vec;
      for (uint32_t v0 = 0; v0 < row_vecs; v0 += G * kUnroll) {  // the order of block_distance
        step_t part = 0;
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
          const uint32_t v = v0 + u * G + lane;
          part += v < row_vecs ? p[v] : (step_t)0;
        }
        acc += (acc_t)part;
      }
      if constexpr (SPLIT) {
        for (uint32_t j = head + row_vecs * EPV + lane; j < block_len; j += G) acc += (acc_t)terms[e_lo + j];
      }
      acc = group_sum<G>(acc);
      if (lane == 0) {
        const uint64_t row = row0 + r;
        if constexpr (DT == DT_I32)
          ((long long*)scores)[row] = (long long)acc;
        else if constexpr (is_tv(DT))
          ((float*)scores)[row] = (float)(0.5 * acc * (double)row_weight[r]);
        else
          ((float*)scores)[row] = (float)acc;
      }
    }
    __syncthreads();  // the next chunk overwrites steps and terms
  }
}

// Row lengths the run-of-rows kernel takes: whole 16-byte steps from 32 to kFlatRowBytes
// bytes (longer ones do as well with a group per row); any other length up to
// kFlatSplitRowBytes whose chunks can start on 16-byte boundaries.  g is the group size the
// listed walk would use - the kernel adds in its order and has G up to 64.  Weighted rows
// (total variation) keep their weights in LDS, which holds them for rows of 32 bytes or more.
static bool flat_rows_fit(bool tv, uint64_t row_bytes, int g) {
  if (g > 64 || (uint64_t)g * kUnroll * 16 < row_bytes) return false;
  if (row_bytes % 16 == 0) return row_bytes >= 32 && row_bytes <= kFlatRowBytes;
  return row_bytes <= kFlatSplitRowBytes && (!tv || row_bytes >= 32) && run_chunk_rows(row_bytes, kFlatVecs) > 0;
}

template <int DT, int G, bool SPLIT>
static void launch_scores_flat(const scar_layout* l, const void* x, const void* c, void* scores,
                               const float* weights, hipStream_t st) {
  constexpr int E = elem_bytes(DT);
  const uint32_t n_rows = (uint32_t)(l->n_elems / l->block_len);
  const uint32_t chunk_rows = run_chunk_rows((uint64_t)l->block_len * E, kFlatVecs);
  const uint32_t n_chunks = (n_rows + chunk_rows - 1) / chunk_rows;
  // five workgroups per compute unit (32 KiB of LDS each, part of it unused) are the best
  // measured: 2.7 M rows of 400 bytes 334 us with eight, 314 us with five or four
  const size_t used = kFlatVecs * sizeof(typename StepSum<DT>::type) + (is_tv(DT) ? kFlatVecs * 2 : 0) +
                      (SPLIT ? kFlatVecs * 16 / E * sizeof(typename ElemTerm<DT>::type) : 0) + 256;
  const size_t lds = used < 32 * 1024 ? 32 * 1024 - used : 0;
  launch((k_block_scores_flat<DT, G, SPLIT>), dim3(xcd_grid(n_chunks, kScoreGridCap)), dim3(kWG),
                     lds, st, (const char*)x, (const char*)c, scores, l->block_len, n_rows, chunk_rows,
                     n_chunks, weights);
  const uint64_t done = (uint64_t)n_rows * l->block_len;
  if (done < l->n_elems) {  // a short last block: a store of one block for the group walk
    const scar_layout last = {l->dtype, l->block_len, l->n_elems - done};
    char* out = (char*)scores + (size_t)n_rows * (DT == DT_I32 ? 8 : 4);
    launch_scores<DT, G>(&last, (const char*)x + done * E, (const char*)c + done * E, out, 1, !SPLIT,
                         weights ? weights + n_rows : nullptr, nullptr, 0, st);
  }
}

template <int DT>
static bool dispatch_scores_flat(int g, bool split, const scar_layout* l, const void* x, const void* c,
                                 void* scores, const float* weights, hipStream_t st) {
#define SCAR_FLAT(G)                                                         \
  case G:                                                                    \
    if (split)                                                               \
      launch_scores_flat<DT, G, true>(l, x, c, scores, weights, st);         \
    else                                                                     \
      launch_scores_flat<DT, G, false>(l, x, c, scores, weights, st);        \
    return true;
  switch (g) {
    SCAR_FLAT(1)
    SCAR_FLAT(2)
    SCAR_FLAT(4)
    SCAR_FLAT(8)
    SCAR_FLAT(16)
    SCAR_FLAT(32)
    SCAR_FLAT(64)
    default: return false;
  }
#undef SCAR_FLAT
}

// ---- a few very long blocks --------------------------------------------------------------
// One workgroup per block leaves most of the chip idle when a store has fewer blocks than the
// chip has room for workgroups (16 shards of 2^26 elements: 16 of 256 compute units).  Such
// blocks are cut into `ppb` pieces of `piece_elems` elements (whole 16-byte steps), one
// workgroup each; a piece's sum goes to partial[entry * ppb + piece] and a second kernel adds a
// block's pieces in a fixed order (reproducible, no atomics).  The pieces depend only on the
// layout, so listed blocks (scar_block_scores_rows) get bit for bit the scores of the full scan.
//
// The partial sums live in a fixed array inside the library's code object (2 MiB per GPU;
// scar_block_scores takes no workspace): calls of this kind on one GPU share it and must not
// overlap.  In host code the array's name is only a handle; its device address is asked for
// once per device and kept.
constexpr uint32_t kGiantMaxPartials = 262144;
constexpr uint32_t kGiantMaxBlocks = 16384;           // more blocks than this fill the chip by themselves
constexpr uint64_t kGiantMinRowBytes = 64 * 1024;     // shorter rows: a workgroup per row is fine
constexpr uint32_t kGiantPieceBytes = 16 * 1024;      // per stream and workgroup, at least: one round of loads
static __device__ __align__(256) unsigned long long giant_partials[kGiantMaxPartials];

constexpr int kGiantMaxDevices = 64;
static void* g_giant_ptr[kGiantMaxDevices];
static std::mutex g_giant_mutex;

static void* giant_partials_of_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kGiantMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_giant_mutex);
  if (!g_giant_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(giant_partials)) != hipSuccess) return nullptr;
    g_giant_ptr[dev] = p;
  }
  return g_giant_ptr[dev];
}

template <int DT, bool VEC>
__global__ __launch_bounds__(kWG) void k_giant_pieces(const char* __restrict__ x, const char* __restrict__ c,
                                                      uint64_t n_elems, uint32_t block_len, uint32_t n_blocks,
                                                      uint32_t ppb, uint32_t piece_elems,
                                                      const uint32_t* __restrict__ idx, uint32_t first_entry,
                                                      uint32_t n_entries,
                                                      typename Acc<DT>::type* __restrict__ partial) {
  using acc_t = typename Acc<DT>::type;
  __shared__ acc_t slots[kWG / kWave];
  const uint64_t total = (uint64_t)n_entries * ppb;
  for (uint64_t w = xcd_contiguous_block_id(); w < total; w += gridDim.x) {
    const uint32_t e = (uint32_t)(w / ppb), piece = (uint32_t)(w % ppb);
    const uint64_t b = idx ? idx[first_entry + e] : first_entry + e;
    acc_t acc = 0;
    if (b < n_blocks) {
      const BlockSpan sp = block_span(b, n_elems, block_len, elem_bytes(DT));
      const uint64_t lo = (uint64_t)piece * piece_elems;
      if (lo < sp.len) {
        // each wavefront walks a contiguous quarter of the piece, as the wavefronts of the
        // scan of 4 KiB blocks each walk a block (measured faster than the four striding
        // through the whole piece together)
        const uint32_t len = (uint32_t)(sp.len - lo < piece_elems ? sp.len - lo : piece_elems);
        const uint32_t quarter = piece_elems / (kWG / kWave);
        const uint32_t q0 = (threadIdx.x / kWave) * quarter;
        if (q0 < len) {
          const uint32_t qlen = len - q0 < quarter ? len - q0 : quarter;
          const uint64_t off = sp.byte_off + (lo + q0) * elem_bytes(DT);
          acc = block_distance<DT, kWave, VEC>(x + off, c + off, qlen, threadIdx.x & (kWave - 1));
        }
      }
    }
    acc = workgroup_sum(acc, slots);
    if (threadIdx.x == 0) partial[w] = acc;
  }
}

// The same pieces for the reduced-precision store (float32 x, bfloat16 c): offsets count
// elements, each wavefront's quarter is split into units by its own addresses (mixed_head).
__global__ __launch_bounds__(kWG) void k_giant_pieces_mixed(const float* __restrict__ x,
                                                            const uint16_t* __restrict__ c, uint64_t n_elems,
                                                            uint32_t block_len, uint32_t n_blocks, uint32_t ppb,
                                                            uint32_t piece_elems, const uint32_t* __restrict__ idx,
                                                            uint32_t first_entry, uint32_t n_entries,
                                                            double* __restrict__ partial) {
  __shared__ double slots[kWG / kWave];
  const uint64_t total = (uint64_t)n_entries * ppb;
  for (uint64_t w = xcd_contiguous_block_id(); w < total; w += gridDim.x) {
    const uint32_t e = (uint32_t)(w / ppb), piece = (uint32_t)(w % ppb);
    const uint64_t b = idx ? idx[first_entry + e] : first_entry + e;
    double acc = 0;
    if (b < n_blocks) {
      const BlockSpan sp = block_span(b, n_elems, block_len, 1);  // byte_off = element offset
      const uint64_t lo = (uint64_t)piece * piece_elems;
      if (lo < sp.len) {
        const uint32_t len = (uint32_t)(sp.len - lo < piece_elems ? sp.len - lo : piece_elems);
        const uint32_t quarter = piece_elems / (kWG / kWave);
        const uint32_t q0 = (threadIdx.x / kWave) * quarter;
        if (q0 < len) {
          const uint32_t qlen = len - q0 < quarter ? len - q0 : quarter;
          const float* xb = x + sp.byte_off + lo + q0;
          const uint16_t* cb = c + sp.byte_off + lo + q0;
          acc = mixed_distance<kWave>(xb, cb, qlen, mixed_head(xb, cb, qlen), threadIdx.x & (kWave - 1));
        }
      }
    }
    acc = workgroup_sum(acc, slots);
    if (threadIdx.x == 0) partial[w] = acc;
  }
}

constexpr int kGiantFinishThreads = 1024;
template <int DT>
__global__ __launch_bounds__(kGiantFinishThreads) void k_giant_finish(
    const typename Acc<DT>::type* __restrict__ partial, uint32_t ppb, uint32_t n_blocks,
    const uint32_t* __restrict__ idx, uint32_t first_entry, const float* __restrict__ weights,
    void* __restrict__ scores) {
  using acc_t = typename Acc<DT>::type;
  constexpr int T = kGiantFinishThreads;
  __shared__ acc_t slots[T / kWave];
  const uint32_t e = blockIdx.x;
  const uint64_t b = idx ? idx[first_entry + e] : first_entry + e;
  if (b >= n_blocks) return;
  const acc_t* mine = partial + (uint64_t)e * ppb;
  acc_t acc = 0;
  uint32_t p = threadIdx.x;
  for (; p + 7 * T < ppb; p += 8 * T) {  // eight loads in flight, added in index order
    acc_t t[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) t[u] = mine[p + u * T];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc += t[u];
  }
  for (; p < ppb; p += T) acc += mine[p];
  acc = workgroup_sum<T>(acc, slots);
  if (threadIdx.x == 0) {
    if constexpr (DT == DT_I32)
      ((long long*)scores)[b] = (long long)acc;
    else if constexpr (is_tv(DT))
      ((float*)scores)[b] = (float)(0.5 * acc * (double)(weights ? weights[b] : 1.f));
    else
      ((float*)scores)[b] = (float)acc;
  }
}

// The same sums for blocks of few pieces (up to kGiantWavePieces): a wavefront per block instead
// of a workgroup of 1,024 threads, which 16,384 blocks of four pieces each would keep busy for
// longer than the scan of their data.  Which of the two kernels adds a block's pieces depends on
// the layout alone, so listed and full scans still agree bit for bit.
constexpr uint32_t kGiantWavePieces = 512;
template <int DT>
__global__ __launch_bounds__(kWG) void k_giant_finish_wave(
    const typename Acc<DT>::type* __restrict__ partial, uint32_t ppb, uint32_t n_blocks,
    const uint32_t* __restrict__ idx, uint32_t first_entry, uint32_t n_entries,
    const float* __restrict__ weights, void* __restrict__ scores) {
  using acc_t = typename Acc<DT>::type;
  const uint32_t e = blockIdx.x * (kWG / kWave) + threadIdx.x / kWave;
  if (e >= n_entries) return;
  const uint64_t b = idx ? idx[first_entry + e] : first_entry + e;
  if (b >= n_blocks) return;
  const acc_t* mine = partial + (uint64_t)e * ppb;
  const uint32_t lane = threadIdx.x & (kWave - 1);
  acc_t acc = 0;
  for (uint32_t p = lane; p < ppb; p += kWave) acc += mine[p];
  acc = group_sum<kWave>(acc);
  if (lane == 0) {
    if constexpr (DT == DT_I32)
      ((long long*)scores)[b] = (long long)acc;
    else if constexpr (is_tv(DT))
      ((float*)scores)[b] = (float)(0.5 * acc * (double)(weights ? weights[b] : 1.f));
    else
      ((float*)scores)[b] = (float)acc;
  }
}

// True if the layout is scored by pieces; ppb / piece_elems receive the cut.
static bool giant_geometry(const scar_layout* l, int eb, uint32_t n_blocks, uint32_t* ppb, uint32_t* piece_elems) {
  const uint64_t row_bytes = (uint64_t)l->block_len * eb;
  if (n_blocks == 0 || n_blocks > kGiantMaxBlocks || row_bytes < kGiantMinRowBytes) return false;
  uint64_t pieces = (row_bytes + kGiantPieceBytes - 1) / kGiantPieceBytes;
  const uint64_t room = kGiantMaxPartials / n_blocks;
  if (pieces > room) pieces = room;
  // whole 16-byte steps per piece, so that every piece starts as aligned as its block does
  const uint64_t per = (uint64_t)(kWG / kWave) * 16 / eb;  // and each wavefront's quarter as well
  uint64_t pe = ((uint64_t)l->block_len + pieces - 1) / pieces;
  pe = (pe + per - 1) / per * per;
  *piece_elems = (uint32_t)pe;
  *ppb = (uint32_t)(((uint64_t)l->block_len + pe - 1) / pe);
  return true;
}

// MIXED: float32 x against a bfloat16 c (DT = DT_F32 for the sums and the scores).
template <int DT, bool MIXED = false>
static int launch_giant(const scar_layout* l, const void* x, const void* c, void* scores, uint32_t n_blocks,
                        bool vec, const float* weights, const uint32_t* idx, uint32_t n_idx, uint32_t ppb,
                        uint32_t piece_elems, hipStream_t st) {
  using acc_t = typename Acc<DT>::type;
  acc_t* partial = (acc_t*)giant_partials_of_current_device();
  if (!partial) return SCAR_ERR_DEVICE;
  const uint32_t n_items = idx ? n_idx : n_blocks;
  const uint32_t per_launch = kGiantMaxPartials / ppb;  // >= n_blocks by construction
  for (uint32_t first = 0; first < n_items; first += per_launch) {
    const uint32_t n_entries = n_items - first < per_launch ? n_items - first : per_launch;
    const uint64_t total = (uint64_t)n_entries * ppb;
    const uint32_t grid = xcd_grid(total, kScoreGridCap);
    const size_t lds = stream_lds_bytes(total, (MIXED ? 24 : 2 * 16) * kWG * kUnroll);
    if constexpr (MIXED)
      launch(k_giant_pieces_mixed, dim3(grid), dim3(kWG), lds, st, (const float*)x, (const uint16_t*)c, l->n_elems,
             l->block_len, n_blocks, ppb, piece_elems, idx, first, n_entries, (double*)partial);
    else if (vec)
      launch((k_giant_pieces<DT, true>), dim3(grid), dim3(kWG), lds, st, (const char*)x, (const char*)c,
             l->n_elems, l->block_len, n_blocks, ppb, piece_elems, idx, first, n_entries, partial);
    else
      launch((k_giant_pieces<DT, false>), dim3(grid), dim3(kWG), lds, st, (const char*)x, (const char*)c,
             l->n_elems, l->block_len, n_blocks, ppb, piece_elems, idx, first, n_entries, partial);
    if (ppb <= kGiantWavePieces)
      launch((k_giant_finish_wave<DT>), dim3((n_entries + kWG / kWave - 1) / (kWG / kWave)), dim3(kWG), 0, st,
             (const acc_t*)partial, ppb, n_blocks, idx, first, n_entries, weights, scores);
    else
      launch((k_giant_finish<DT>), dim3(n_entries), dim3(kGiantFinishThreads), 0, st, (const acc_t*)partial, ppb,
             n_blocks, idx, first, weights, scores);
  }
  return launch_status();
}

// Scores of a reduced-precision store that is a few very long blocks; false if the layout is
// not of that kind (then nothing has been enqueued and *status is untouched).
bool mixed_giant_scores(const scar_layout* l, uint32_t n_blocks, const void* x, const void* c,
                        const uint32_t* idx, uint32_t n_idx, void* scores, hipStream_t st, int* status) {
  uint32_t ppb = 0, piece_elems = 0;
  if (!giant_geometry(l, 4, n_blocks, &ppb, &piece_elems)) return false;
  *status = launch_giant<DT_F32, true>(l, x, c, scores, n_blocks, false, nullptr, idx, n_idx, ppb, piece_elems, st);
  return true;
}

template <int DT>
static void dispatch_scores(int g, const scar_layout* l, const void* x, const void* c, void* scores,
                            uint32_t n_blocks, bool vec, const float* weights, const uint32_t* idx,
                            uint32_t n_idx, hipStream_t st) {
  switch (g) {
    case 1: launch_scores<DT, 1>(l, x, c, scores, n_blocks, vec, weights, idx, n_idx, st); break;
    case 2: launch_scores<DT, 2>(l, x, c, scores, n_blocks, vec, weights, idx, n_idx, st); break;
    case 4: launch_scores<DT, 4>(l, x, c, scores, n_blocks, vec, weights, idx, n_idx, st); break;
    case 8: launch_scores<DT, 8>(l, x, c, scores, n_blocks, vec, weights, idx, n_idx, st); break;
    case 16: launch_scores<DT, 16>(l, x, c, scores, n_blocks, vec, weights, idx, n_idx, st); break;
    case 32: launch_scores<DT, 32>(l, x, c, scores, n_blocks, vec, weights, idx, n_idx, st); break;
    case 64: launch_scores<DT, 64>(l, x, c, scores, n_blocks, vec, weights, idx, n_idx, st); break;
    default: launch_scores<DT, 256>(l, x, c, scores, n_blocks, vec, weights, idx, n_idx, st); break;
  }
}

}  // namespace scar

using namespace scar;

// Shared body of scar_block_scores (tv = false), scar_tv_block_scores and, with a list of
// blocks (listed = true), scar_block_scores_rows.
static int block_scores(bool tv, bool listed, const scar_layout* layout, const void* x, const void* c,
                        const float* weights, const uint32_t* idx, uint32_t n_idx, void* scores,
                        void* stream) {
  const uint64_t nb = layout_blocks(layout);
  if (nb == UINT64_MAX) return SCAR_ERR_INVALID_ARG;
  if (tv && layout->dtype != SCAR_F32 && layout->dtype != SCAR_BF16) return SCAR_ERR_UNSUPPORTED;
  if (nb == 0 || (listed && n_idx == 0)) return SCAR_OK;
  if (listed && (!idx || !aligned(idx, 4))) return SCAR_ERR_INVALID_ARG;
  if (!listed) idx = nullptr;
  if (layout->dtype == SCAR_F32_BF16C)
    return mixed_block_scores(layout, (uint32_t)nb, x, c, idx, n_idx, scores, (hipStream_t)stream);
  const int eb = host_elem_bytes(layout->dtype);
  if (!x || !c || !scores || !aligned(x, eb) || !aligned(c, eb) || !aligned(weights, 4) ||
      !aligned(scores, layout->dtype == SCAR_I32 ? 8 : 4))
    return SCAR_ERR_INVALID_ARG;
  const bool vec = aligned(x, 16) && aligned(c, 16) && ((uint64_t)layout->block_len * eb) % 16 == 0;
  const uint64_t row_bytes = (uint64_t)layout->block_len * eb;
  // Four loads per lane and stream, except for short rows that are not whole 128-byte lines:
  // there every 16-byte step of a group straddles cache lines, and a wider group with two
  // steps per lane asks for each line half as often (165,000 rows of 400 bytes: 29.6 -> 24.4 us).
  const int per_lane = (vec && row_bytes % 128 != 0 && row_bytes <= 1024) ? 2 : 4;
  int g = pick_group(layout->block_len, eb, co_aligned(x, c), per_lane, false);
  // rows of more than 96 steps: a whole wavefront with two loads per lane instead of half of one
  // with four (2^28 elements in rows of 2,000 bytes: bf16 179 -> 162 us, f32 331 -> 309 us;
  // rows of 1,280 bytes would lose, 80 steps leave too many of the 128 slots empty)
  if (g == 32 && vec && row_bytes > 1536) g = 64;
  hipStream_t st = (hipStream_t)stream;
  const uint32_t n = (uint32_t)nb;
  if (!tv && !listed && row_bytes < 16 && aligned(x, 16) && aligned(c, 16)) {  // rows of 2, 4 or 8 bytes
    bool done = false;
    switch (layout->dtype) {
      case SCAR_F32: done = launch_scores_tiny<DT_F32>(layout, x, c, scores, st); break;
      case SCAR_BF16: done = launch_scores_tiny<DT_BF16>(layout, x, c, scores, st); break;
      default: done = launch_scores_tiny<DT_I32>(layout, x, c, scores, st); break;
    }
    if (done) return launch_status();
  }
  // a few very long blocks: cut into pieces, many workgroups per block
  uint32_t ppb = 0, piece_elems = 0;
  if (giant_geometry(layout, eb, n, &ppb, &piece_elems)) {
    const bool vec_pieces = aligned(x, 16) && aligned(c, 16) && row_bytes % 16 == 0;
    if (tv && layout->dtype == SCAR_F32)
      return launch_giant<DT_F32_TV>(layout, x, c, scores, n, vec_pieces, weights, idx, n_idx, ppb, piece_elems, st);
    if (tv) return launch_giant<DT_BF16_TV>(layout, x, c, scores, n, vec_pieces, weights, idx, n_idx, ppb, piece_elems, st);
    switch (layout->dtype) {
      case SCAR_F32: return launch_giant<DT_F32>(layout, x, c, scores, n, vec_pieces, nullptr, idx, n_idx, ppb, piece_elems, st);
      case SCAR_BF16: return launch_giant<DT_BF16>(layout, x, c, scores, n, vec_pieces, nullptr, idx, n_idx, ppb, piece_elems, st);
      default: return launch_giant<DT_I32>(layout, x, c, scores, n, vec_pieces, nullptr, idx, n_idx, ppb, piece_elems, st);
    }
  }
  // many short rows of an aligned store: read as runs of whole rows
  const bool split = row_bytes % 16 != 0;
  if (!listed && aligned(x, 16) && aligned(c, 16) && n >= kFlatMinRows && flat_rows_fit(tv, row_bytes, g)) {
    bool done = false;
    if (tv && layout->dtype == SCAR_F32) done = dispatch_scores_flat<DT_F32_TV>(g, split, layout, x, c, scores, weights, st);
    else if (tv) done = dispatch_scores_flat<DT_BF16_TV>(g, split, layout, x, c, scores, weights, st);
    else if (layout->dtype == SCAR_F32) done = dispatch_scores_flat<DT_F32>(g, split, layout, x, c, scores, nullptr, st);
    else if (layout->dtype == SCAR_BF16) done = dispatch_scores_flat<DT_BF16>(g, split, layout, x, c, scores, nullptr, st);
    else done = dispatch_scores_flat<DT_I32>(g, split, layout, x, c, scores, nullptr, st);
    if (done) return launch_status();
  }
  if (tv) {
    if (layout->dtype == SCAR_F32)
      dispatch_scores<DT_F32_TV>(g, layout, x, c, scores, n, vec, weights, idx, n_idx, st);
    else
      dispatch_scores<DT_BF16_TV>(g, layout, x, c, scores, n, vec, weights, idx, n_idx, st);
    return launch_status();
  }
  switch (layout->dtype) {
    case SCAR_F32: dispatch_scores<DT_F32>(g, layout, x, c, scores, n, vec, nullptr, idx, n_idx, st); break;
    case SCAR_BF16: dispatch_scores<DT_BF16>(g, layout, x, c, scores, n, vec, nullptr, idx, n_idx, st); break;
    default: dispatch_scores<DT_I32>(g, layout, x, c, scores, n, vec, nullptr, idx, n_idx, st); break;
  }
  return launch_status();
}

extern "C" int scar_block_scores(const scar_layout* layout, const void* x, const void* c,
                                 void* scores, void* stream) {
  return block_scores(false, false, layout, x, c, nullptr, nullptr, 0, scores, stream);
}

extern "C" int scar_tv_block_scores(const scar_layout* layout, const void* x, const void* c,
                                    const float* weights, float* scores, void* stream) {
  return block_scores(true, false, layout, x, c, weights, nullptr, 0, scores, stream);
}

extern "C" int scar_block_scores_rows(const scar_layout* layout, const void* x, const void* c,
                                      const uint32_t* idx, uint32_t n_idx, void* scores, void* stream) {
  return block_scores(false, true, layout, x, c, nullptr, idx, n_idx, scores, stream);
}

