// Index-driven row kernels: scar_checkpoint_commit (checkpoint step 4 of Section 4.3),
// scar_partial_recover with the fused norm (Section 4.1, Appendix A.3) and
// scar_perturbation_norm.
//
// Each group of G lanes takes one entry of the index list, finds its block and moves or
// measures it with 16-byte accesses.  The norm is reduced in two deterministic stages:
// one partial sum per workgroup (float64, or exact int64 for integer tables), then a
// single workgroup adds the partials in a fixed order.
#include "scar_device.hpp"
#include "scar_host.hpp"

namespace scar {

// Long rows are handed out in pieces of kPieceBytes, so that a few long rows fill the chip as
// well as many short ones (and every piece takes the loop-free path): the grid's y dimension
// runs over the pieces of a row, its x dimension over the index list.  pieces == 1: whole rows
// of any length.
struct RowPiece {
  uint64_t byte_off;   // of the piece within x and c
  uint32_t row_off;    // of the piece within its row, in bytes
  uint32_t len;        // elements
};

// False if there is nothing there (index out of range, piece beyond a short last block).
template <int E>
__device__ __forceinline__ bool row_piece(uint32_t b, uint32_t piece, uint32_t pieces, uint32_t n_blocks,
                                          uint64_t n_elems, uint32_t block_len, RowPiece* out) {
  if (b >= n_blocks) return false;
  const BlockSpan sp = block_span(b, n_elems, block_len, E);
  constexpr uint32_t kPieceElems = kPieceBytes / E;
  const uint32_t first = piece * kPieceElems;
  if (first >= sp.len) return false;
  uint32_t len = sp.len - first;
  if (pieces > 1 && len > kPieceElems) len = kPieceElems;
  *out = {sp.byte_off + (uint64_t)first * E, first * (uint32_t)E, len};
  return true;
}

// c_b <- x_b (and staging row i <- x_b) for b = idx[i].
template <int G, typename W>
__global__ __launch_bounds__(kWG) void k_commit(const char* __restrict__ x, char* __restrict__ c,
                                                const uint32_t* __restrict__ idx, uint32_t n_idx,
                                                char* __restrict__ staging, uint64_t n_elems,
                                                uint32_t block_len, uint32_t n_blocks, uint32_t pieces,
                                                bool vec, bool vec_staging) {
  constexpr int GPW = (G == 256) ? 1 : kWG / G;
  const int lane = (G == 256) ? threadIdx.x : (threadIdx.x & (G - 1));
  const uint32_t grp = (G == 256) ? 0 : threadIdx.x / G;
  const GridSlot slot = row_grid_slot(((uint64_t)n_idx + GPW - 1) / GPW);
  for (uint32_t piece = slot.y; piece < pieces; piece += gridDim.y) {
    for (uint64_t i = (uint64_t)slot.x * GPW + grp; i < n_idx;
         i += (uint64_t)gridDim.x * GPW) {
      RowPiece rp;
      if (!row_piece<sizeof(W)>(idx[i], piece, pieces, n_blocks, n_elems, block_len, &rp)) continue;
      char* st = staging ? staging + i * (uint64_t)block_len * sizeof(W) + rp.row_off : nullptr;
      block_copy<G, W>(x + rp.byte_off, c + rp.byte_off, st, rp.len * (uint32_t)sizeof(W), lane, vec,
                       vec_staging);
    }
  }
}

// One row (or one piece of a long row) of the recovery / norm pass, spread over a group of G
// lanes: acc gets this lane's share of sum (c - x)^2 or sum |c - x| (NORM), then x <- c (STORE).
//   VEC: both rows start 16-byte aligned and hold at most G 16-byte steps - the host sizes G
//   and the pieces for that - plus a tail that only the store's last, short block can have:
//   one load per stream and lane, no loop.  Otherwise the row is split as row_split says.
template <int DT, int G, bool STORE, bool NORM, bool VEC>
__device__ __forceinline__ void recover_row(char* xb, const char* cb, uint32_t len, int lane,
                                            typename Acc<DT>::type& acc) {
  constexpr int E = elem_bytes(DT);
  constexpr int EPV = 16 / E;
  using word_t = typename std::conditional<E == 4, uint32_t, uint16_t>::type;
  auto element = [&](uint32_t j) {
    if (NORM) accumulate_elem<DT>(acc, cb, xb, j);
    if (STORE) ((word_t*)xb)[j] = ((const word_t*)cb)[j];
  };
  if constexpr (VEC) {
    const uint32_t nvec = len / EPV;
    if ((uint32_t)lane < nvec) {
      uint4 cv[1], xv[1];
      cv[0] = load_stream((const uint4*)cb + lane);
      if (NORM) {
        xv[0] = load_stream((const uint4*)xb + lane);
        accumulate_vec<DT, 1>(acc, cv, xv);
      }
      if (STORE) store_stream((uint4*)xb + lane, cv[0]);
    }
    for (uint32_t j = nvec * EPV + lane; j < len; j += G) element(j);
    return;
  }
  const RowSplit rs = row_split<E>(xb, cb, len);
  const uint32_t head = rs.head, nvec = rs.nvec;
  const uint32_t tail0 = head + nvec * EPV;
  // The few elements before and after the 16-byte steps are fetched together with the first
  // steps - one round trip to memory for a short row, not three - when the group has a lane
  // for each of them; a row that is walked element by element (head == len) loops instead.
  const bool ends_in_lanes = G >= EPV && head < (uint32_t)EPV;
  const bool has_head = ends_in_lanes && (uint32_t)lane < head, has_tail = ends_in_lanes && tail0 + lane < len;
  word_t hc = 0, hx = 0, tc = 0, tx = 0;
  if (has_head) {
    hc = ((const word_t*)cb)[lane];
    if (NORM) hx = ((const word_t*)xb)[lane];
  }
  if (has_tail) {
    tc = ((const word_t*)cb)[tail0 + lane];
    if (NORM) tx = ((const word_t*)xb)[tail0 + lane];
  }
  if (!ends_in_lanes)
    for (uint32_t j = lane; j < head; j += G) element(j);
  if (NORM && has_head) accumulate_elem<DT>(acc, (const char*)&hc, (const char*)&hx, 0);
  uint4* xvp = (uint4*)(xb + (size_t)head * E);
  const uint4* cvp = (const uint4*)(cb + (size_t)head * E);
  for (uint32_t v0 = 0; v0 < nvec; v0 += G * kUnroll) {
    uint4 xv[kUnroll], cv[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const uint32_t v = v0 + u * G + lane;
      if (v < nvec) {
        cv[u] = load_stream(cvp + v);
        xv[u] = NORM ? load_stream((const uint4*)xvp + v) : make_uint4(0, 0, 0, 0);
      } else {
        cv[u] = make_uint4(0, 0, 0, 0);
        xv[u] = make_uint4(0, 0, 0, 0);
      }
    }
    if (NORM) accumulate_vec<DT, kUnroll>(acc, cv, xv);
    if (STORE) {
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const uint32_t v = v0 + u * G + lane;
        if (v < nvec) store_stream(xvp + v, cv[u]);
      }
    }
  }
  if (NORM && has_tail) accumulate_elem<DT>(acc, (const char*)&tc, (const char*)&tx, 0);
  if (STORE) {  // after the steps: measured faster here than in address order (the copy kernel differs)
    if (has_head) ((word_t*)xb)[lane] = hc;
    if (has_tail) ((word_t*)xb)[tail0 + lane] = tc;
  }
  if (!ends_in_lanes)
    for (uint32_t j = tail0 + lane; j < len; j += G) element(j);
}

// Recovery and/or norm over the blocks idx[0..n_idx) (idx == NULL: blocks 0..n_idx).
//   STORE: x_b <- c_b after the block has been measured.
//   NORM:  partial[blockIdx.x] <- this workgroup's share of sum (c - x)^2 or sum |c - x|.
//   weights (total-variation kinds only): per-block factors of the sum, NULL = 1.
//   T:     threads per workgroup, T / G groups.  The second launch bound asks for 8 wavefronts
//          per SIMD when T = 1,024 (at most 64 registers), so that two such workgroups fit a
//          compute unit; with one more register the kernel runs a quarter slower.  Long index lists run with 1,024 threads: a
//          workgroup that has to come back for a second entry waits a full memory round trip
//          in between (131,072 rows of 4 KiB: 298 us with two entries per group, 283 us with
//          one), and a quarter of the workgroups also means a quarter of the partial sums.
template <int DT, int G, int T, bool STORE, bool NORM, bool VEC>
__global__ __launch_bounds__(T, T / 128) void k_recover(char* __restrict__ x, const char* __restrict__ c,
                                               const uint32_t* __restrict__ idx, uint32_t n_idx,
                                               uint64_t n_elems, uint32_t block_len,
                                               uint32_t n_blocks, uint32_t pieces, bool packed,
                                               typename Acc<DT>::type* __restrict__ partial,
                                               const float* __restrict__ weights) {
  constexpr int GPW = T / G;
  constexpr int E = elem_bytes(DT);
  using acc_t = typename Acc<DT>::type;
  const int lane = threadIdx.x & (G - 1);
  const uint32_t grp = threadIdx.x / G;
  __shared__ acc_t slots[T / kWave];
  acc_t acc = 0;

  const GridSlot slot = row_grid_slot(((uint64_t)n_idx + GPW - 1) / GPW);
  for (uint32_t piece = slot.y; piece < pieces; piece += gridDim.y) {
    for (uint64_t i = (uint64_t)slot.x * GPW + grp; i < n_idx;
         i += (uint64_t)gridDim.x * GPW) {
      const uint32_t b = idx ? idx[i] : (uint32_t)i;
      RowPiece rp;
      if (!row_piece<E>(b, piece, pieces, n_blocks, n_elems, block_len, &rp)) continue;
      // packed: c holds only the listed blocks, row i = block idx[i] (rows read back from storage)
      const char* cb = packed ? c + i * (uint64_t)block_len * E + rp.row_off : c + rp.byte_off;
      if constexpr (is_tv(DT)) {  // each row's share counts with the row's weight
        const float w = weights ? weights[b] : 1.f;  // asked for before the row, used after it
        acc_t row = 0;
        recover_row<DT, G, STORE, NORM, VEC>(x + rp.byte_off, cb, rp.len, lane, row);
        acc += (double)w * row;
      } else {
        recover_row<DT, G, STORE, NORM, VEC>(x + rp.byte_off, cb, rp.len, lane, acc);
      }
    }
  }
  if (NORM) {
    acc = workgroup_sum<T>(acc, slots);
    if (threadIdx.x == 0) partial[blockIdx.y * gridDim.x + blockIdx.x] = acc;
  }
}

// The norm alone over a long list (nothing stored), with the result of k_recover<DT, G, 1024,
// false, true, true> bit for bit - the norm fused into the recovery must equal the norm taken
// beforehand - but with the loads of the score scan: a workgroup of 256 threads stands in for
// one of 1,024, each wavefront for kVirtual of the wide kernel's wavefronts.  A lane asks for
// the 16-byte steps of its kVirtual virtual lanes before it uses the first (4 loads per stream
// in flight instead of 1), keeps one sum per virtual lane, reduces each virtual wavefront on
// its own and leaves the 16 sums in the slots in the wide kernel's order.  Launched with that
// kernel's grid, so the partial sums are the same ones.  (131,072 rows of 4 KiB: 240 -> 191 us
// with the final sum; limiting the workgroups per compute unit, good for the scans, costs 40 %
// here: every workgroup first waits for its index entries.)
constexpr int kVirtual = 4;
template <int DT, int G>
__global__ __launch_bounds__(kWG) void k_norm_wide(const char* __restrict__ x, const char* __restrict__ c,
                                                   const uint32_t* __restrict__ idx, uint32_t n_idx,
                                                   uint64_t n_elems, uint32_t block_len,
                                                   uint32_t n_blocks, uint32_t pieces, bool packed,
                                                   typename Acc<DT>::type* __restrict__ partial,
                                                   const float* __restrict__ weights) {
  constexpr int T = kWG * kVirtual;  // threads of the kernel this one stands in for
  constexpr int GPW = T / G;
  constexpr int E = elem_bytes(DT);
  constexpr int EPV = 16 / E;
  using acc_t = typename Acc<DT>::type;
  __shared__ acc_t slots[T / kWave];
  const uint32_t wave = threadIdx.x / kWave, in_wave = threadIdx.x & (kWave - 1);
  acc_t acc[kVirtual];
#pragma unroll
  for (int q = 0; q < kVirtual; ++q) acc[q] = 0;

  const GridSlot slot = row_grid_slot(((uint64_t)n_idx + GPW - 1) / GPW);
  for (uint32_t piece = slot.y; piece < pieces; piece += gridDim.y) {
    for (uint64_t i0 = (uint64_t)slot.x * GPW; i0 < n_idx; i0 += (uint64_t)gridDim.x * GPW) {
      const char* xb[kVirtual];
      const char* cb[kVirtual];
      uint32_t len[kVirtual], lane[kVirtual];
      float w[kVirtual];
      uint4 cv[kVirtual][1], xv[kVirtual][1];
      bool on[kVirtual], has_step[kVirtual];
#pragma unroll
      for (int q = 0; q < kVirtual; ++q) {
        const uint32_t vt = (wave * kVirtual + q) * kWave + in_wave;  // thread of the wide workgroup
        lane[q] = vt & (G - 1);
        const uint64_t i = i0 + vt / G;
        on[q] = false, has_step[q] = false, w[q] = 1.f;
        if (i >= n_idx) continue;
        const uint32_t b = idx ? idx[i] : (uint32_t)i;
        RowPiece rp;
        if (!row_piece<E>(b, piece, pieces, n_blocks, n_elems, block_len, &rp)) continue;
        on[q] = true;
        xb[q] = x + rp.byte_off;
        cb[q] = packed ? c + i * (uint64_t)block_len * E + rp.row_off : c + rp.byte_off;
        len[q] = rp.len;
        if constexpr (is_tv(DT))
          if (weights) w[q] = weights[b];
        has_step[q] = lane[q] < rp.len / EPV;
        if (has_step[q]) {
          cv[q][0] = load_stream((const uint4*)cb[q] + lane[q]);
          xv[q][0] = load_stream((const uint4*)xb[q] + lane[q]);
        }
      }
#pragma unroll
      for (int q = 0; q < kVirtual; ++q) {
        if (!on[q]) continue;
        // as k_recover adds: the step, then what a short last block has left - into the running
        // sum, or (total variation) into the row's own sum, which counts with the row's weight
        acc_t row = 0;
        acc_t& into = is_tv(DT) ? row : acc[q];
        if (has_step[q]) accumulate_vec<DT, 1>(into, cv[q], xv[q]);
        for (uint32_t j = len[q] / EPV * EPV + lane[q]; j < len[q]; j += G) accumulate_elem<DT>(into, cb[q], xb[q], j);
        if constexpr (is_tv(DT)) acc[q] += (double)w[q] * row;
      }
    }
  }
#pragma unroll
  for (int q = 0; q < kVirtual; ++q) {
    const acc_t v = group_sum<kWave>(acc[q]);
    if (in_wave == 0) slots[wave * kVirtual + q] = v;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    acc_t total = slots[0];
#pragma unroll
    for (int v = 1; v < T / kWave; ++v) total += slots[v];
    partial[blockIdx.y * gridDim.x + blockIdx.x] = total;
  }
}

// The norm over the whole store with nothing stored (the perturbation a traditional full
// recovery would cause, Appendix A.3): the sum does not depend on where the blocks begin, so
// this is one flat two-stream reduction - kUnroll 16-byte loads per lane and stream in flight,
// as in the score scan, instead of one row per group.  Each 16-byte step is summed in float32
// and folded into float64 on its own, as the row walk does it.  Needs 16-byte aligned bases;
// the elements after the last whole step go to the first workgroup.
template <int DT>
__global__ __launch_bounds__(kWG) void k_norm_all(const char* __restrict__ x, const char* __restrict__ c,
                                                  uint64_t n_elems,
                                                  typename Acc<DT>::type* __restrict__ partial) {
  constexpr int EPV = 16 / elem_bytes(DT);
  using acc_t = typename Acc<DT>::type;
  __shared__ acc_t slots[kWG / kWave];
  const uint64_t nvec = n_elems / EPV;
  acc_t acc = 0;
  for (uint64_t v0 = (uint64_t)xcd_contiguous_block_id() * (kWG * kUnroll); v0 < nvec;
       v0 += (uint64_t)gridDim.x * (kWG * kUnroll)) {
    uint4 cv[kUnroll][1], xv[kUnroll][1];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const uint64_t v = v0 + (uint64_t)u * kWG + threadIdx.x;
      if (v < nvec) {
        cv[u][0] = load_stream((const uint4*)c + v);
        xv[u][0] = load_stream((const uint4*)x + v);
      } else {
        cv[u][0] = make_uint4(0, 0, 0, 0);
        xv[u][0] = make_uint4(0, 0, 0, 0);
      }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) accumulate_vec<DT, 1>(acc, cv[u], xv[u]);
  }
  if (blockIdx.x == 0)
    for (uint64_t j = nvec * EPV + threadIdx.x; j < n_elems; j += kWG) accumulate_elem<DT>(acc, c, x, j);
  acc = workgroup_sum(acc, slots);
  if (threadIdx.x == 0) partial[blockIdx.x] = acc;
}

template <int DT>
static uint32_t launch_norm_all(const scar_layout* l, const void* x, const void* c, void* partial,
                                hipStream_t st) {
  const uint64_t nvec = l->n_elems / (16 / elem_bytes(DT));
  const uint64_t chunks = (nvec + kWG * kUnroll - 1) / (kWG * kUnroll);
  const uint32_t grid = xcd_grid(chunks ? chunks : 1, kMaxNormGrid);
  launch((k_norm_all<DT>), dim3(grid), dim3(kWG), stream_lds_bytes(grid, 2 * 16 * kWG * kUnroll), st,
                     (const char*)x, (const char*)c, l->n_elems, (typename Acc<DT>::type*)partial);
  return grid;
}

// Second stage of the norm: one workgroup of 1024 threads adds n_partial partial sums in
// a fixed order and writes the result.  n_partial == 0 writes zeros.
constexpr int kFinishThreads = 1024;
template <int DT>
__global__ __launch_bounds__(kFinishThreads) void k_norm_finish(
    const typename Acc<DT>::type* __restrict__ partial, uint32_t n_partial, scar_norm* __restrict__ out) {
  using acc_t = typename Acc<DT>::type;
  __shared__ acc_t slots[kFinishThreads / kWave];
  acc_t acc = 0;
  uint32_t i = threadIdx.x;
  for (; i + 15 * kFinishThreads < n_partial; i += 16 * kFinishThreads) {  // 16 loads in flight
    acc_t t[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) t[u] = partial[i + u * kFinishThreads];
#pragma unroll
    for (int u = 0; u < 16; ++u) acc += t[u];
  }
  for (; i < n_partial; i += kFinishThreads) acc += partial[i];
  acc = group_sum<kWave>(acc);
  if ((threadIdx.x & (kWave - 1)) == 0) slots[threadIdx.x / kWave] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    acc_t total = 0;
    for (int w = 0; w < kFinishThreads / kWave; ++w) total += slots[w];
    if constexpr (DT == DT_I32) {
      out->isum = (long long)total;
      out->sum = (double)total;
      out->norm = (double)total;
    } else if constexpr (is_tv(DT)) {  // sum of w_b * 1/2 * sum |c - x|; the norm is that sum
      out->isum = 0;
      out->sum = 0.5 * total;
      out->norm = 0.5 * total;
    } else {
      out->isum = 0;
      out->sum = total;
      out->norm = sqrt(total);
    }
  }
}

template <int G, typename W>
static void launch_commit(const scar_layout* l, const void* x, void* c, const uint32_t* idx,
                          uint32_t n_idx, void* staging, uint32_t n_blocks, uint32_t pieces, bool vec,
                          bool vec_st, hipStream_t st) {
  constexpr int GPW = (G == 256) ? 1 : kWG / G;
  const RowGrid rg = row_grid(((uint64_t)n_idx + GPW - 1) / GPW, pieces, kCopyGridCap);
  launch((k_commit<G, W>), dim3(rg.x, rg.y), dim3(kWG), 0, st, (const char*)x, (char*)c, idx,
                     n_idx, (char*)staging, l->n_elems, l->block_len, n_blocks, pieces, vec, vec_st);
}

template <typename W>
static void dispatch_commit(int g, const scar_layout* l, const void* x, void* c, const uint32_t* idx,
                            uint32_t n_idx, void* staging, uint32_t n_blocks, uint32_t pieces, bool vec,
                            bool vec_st, hipStream_t st) {
#define SCAR_CALL(G) launch_commit<G, W>(l, x, c, idx, n_idx, staging, n_blocks, pieces, vec, vec_st, st); break
  switch (g) {
    case 1: SCAR_CALL(1);
    case 2: SCAR_CALL(2);
    case 4: SCAR_CALL(4);
    case 8: SCAR_CALL(8);
    case 16: SCAR_CALL(16);
    case 32: SCAR_CALL(32);
    case 64: SCAR_CALL(64);
    case 128: SCAR_CALL(128);
    default: SCAR_CALL(256);
  }
#undef SCAR_CALL
}

// Pieces per row for the copy kernels: long rows of a 16-byte-aligned store are cut at every
// kPieceBytes; anything else goes row by row.
static uint32_t row_pieces(const scar_layout* l, int eb, bool vec) {
  const uint64_t row_bytes = (uint64_t)l->block_len * eb;
  return (vec && row_bytes > kPieceBytes) ? (uint32_t)((row_bytes + kPieceBytes - 1) / kPieceBytes) : 1;
}

// Launches the recovery / norm kernel; returns the number of partial sums it writes.
constexpr int kWideWG = 1024;
constexpr uint64_t kWideFrom = 8192;   // workgroups of kWG threads from which kWideWG is used
constexpr uint32_t kWideMinEntries = 64;

template <int DT, int G, int T, bool STORE, bool NORM, bool VEC>
static uint32_t launch_recover_t(const scar_layout* l, void* x, const void* c, const uint32_t* idx,
                                 uint32_t n_idx, uint32_t n_blocks, uint32_t pieces, bool packed,
                                 void* partial, const float* weights, hipStream_t st) {
  constexpr int GPW = T / G;
  const RowGrid rg = row_grid(((uint64_t)n_idx + GPW - 1) / GPW, pieces, kMaxNormGrid);
  const uint32_t grid = rg.x, grid_y = rg.y;
  launch((k_recover<DT, G, T, STORE, NORM, VEC>), dim3(grid, grid_y), dim3(T), 0, st, (char*)x,
                     (const char*)c, idx, n_idx, l->n_elems, l->block_len, n_blocks, pieces, packed,
                     (typename Acc<DT>::type*)partial, weights);
  return grid * grid_y;
}

template <int DT, int G, bool STORE, bool NORM>
static uint32_t launch_recover(const scar_layout* l, void* x, const void* c, const uint32_t* idx,
                               uint32_t n_idx, uint32_t n_blocks, uint32_t pieces, bool vec, bool packed,
                               void* partial, const float* weights, hipStream_t st) {
  if (!vec)
    return launch_recover_t<DT, G, kWG, STORE, NORM, false>(l, x, c, idx, n_idx, n_blocks, pieces, packed, partial, weights, st);
  // (a list shorter than the groups of a few wide workgroups would leave most of them idle)
  if (n_idx >= kWideMinEntries && ((uint64_t)n_idx * pieces * G + kWG - 1) / kWG >= kWideFrom) {
    if constexpr (!STORE && NORM) {  // read-only: the same sums from a kernel with more loads in flight
      static_assert(kWideWG == kWG * kVirtual, "k_norm_wide stands in for the wide kernel");
      constexpr int GPW = kWideWG / G;
      const RowGrid rg = row_grid(((uint64_t)n_idx + GPW - 1) / GPW, pieces, kMaxNormGrid);
      const uint32_t grid = rg.x, grid_y = rg.y;
      launch((k_norm_wide<DT, G>), dim3(grid, grid_y), dim3(kWG),
                         0, st, (const char*)x,
                         (const char*)c, idx, n_idx, l->n_elems, l->block_len, n_blocks, pieces, packed,
                         (typename Acc<DT>::type*)partial, weights);
      return grid * grid_y;
    }
    return launch_recover_t<DT, G, kWideWG, STORE, NORM, true>(l, x, c, idx, n_idx, n_blocks, pieces, packed, partial, weights, st);
  }
  return launch_recover_t<DT, G, kWG, STORE, NORM, true>(l, x, c, idx, n_idx, n_blocks, pieces, packed, partial, weights, st);
}

template <int DT, bool STORE, bool NORM>
static uint32_t dispatch_recover_g(int g, const scar_layout* l, void* x, const void* c,
                                   const uint32_t* idx, uint32_t n_idx, uint32_t n_blocks,
                                   uint32_t pieces, bool vec, bool packed, void* partial,
                                   const float* weights, hipStream_t st) {
#define SCAR_CALL(G) \
  return launch_recover<DT, G, STORE, NORM>(l, x, c, idx, n_idx, n_blocks, pieces, vec, packed, partial, weights, st)
  switch (g) {
    case 1: SCAR_CALL(1);
    case 2: SCAR_CALL(2);
    case 4: SCAR_CALL(4);
    case 8: SCAR_CALL(8);
    case 16: SCAR_CALL(16);
    case 32: SCAR_CALL(32);
    case 64: SCAR_CALL(64);
    case 128: SCAR_CALL(128);
    default: SCAR_CALL(256);
  }
#undef SCAR_CALL
}

// dt: what is measured (a DT_* kind).  The total-variation kinds always measure (NORM).
template <bool STORE, bool NORM>
static uint32_t dispatch_recover(int dt, int g, const scar_layout* l, void* x, const void* c,
                                 const uint32_t* idx, uint32_t n_idx, uint32_t n_blocks, uint32_t pieces,
                                 bool vec, bool packed, void* partial, const float* weights, hipStream_t st) {
  switch (dt) {
    case DT_F32: return dispatch_recover_g<DT_F32, STORE, NORM>(g, l, x, c, idx, n_idx, n_blocks, pieces, vec, packed, partial, nullptr, st);
    case DT_BF16: return dispatch_recover_g<DT_BF16, STORE, NORM>(g, l, x, c, idx, n_idx, n_blocks, pieces, vec, packed, partial, nullptr, st);
    case DT_I32: return dispatch_recover_g<DT_I32, STORE, NORM>(g, l, x, c, idx, n_idx, n_blocks, pieces, vec, packed, partial, nullptr, st);
    case DT_F32_TV:
      if constexpr (NORM) return dispatch_recover_g<DT_F32_TV, STORE, true>(g, l, x, c, idx, n_idx, n_blocks, pieces, vec, packed, partial, weights, st);
      return 0;
    default:
      if constexpr (NORM) return dispatch_recover_g<DT_BF16_TV, STORE, true>(g, l, x, c, idx, n_idx, n_blocks, pieces, vec, packed, partial, weights, st);
      return 0;
  }
}

void launch_finish_tv(const void* partial, uint32_t n_partial, scar_norm* out, hipStream_t st) {
  launch((k_norm_finish<DT_F32_TV>), dim3(1), dim3(kFinishThreads), 0, st, (const double*)partial,
                     n_partial, out);
}

void launch_finish(int32_t dtype, const void* partial, uint32_t n_partial, scar_norm* out,
                          hipStream_t st) {
  if (dtype == SCAR_I32)
    launch((k_norm_finish<DT_I32>), dim3(1), dim3(kFinishThreads), 0, st,
                       (const unsigned long long*)partial, n_partial, out);
  else
    launch((k_norm_finish<DT_F32>), dim3(1), dim3(kFinishThreads), 0, st, (const double*)partial,
                       n_partial, out);
}

// Shared body of scar_partial_recover (store = true) and scar_perturbation_norm, and of their
// total-variation twins (tv = true: float stores only, weights may be NULL).
static int recover_or_norm(bool store, bool packed, bool tv, const scar_layout* layout, void* x,
                           const void* c, const float* weights, const uint32_t* idx, uint32_t n_idx,
                           bool all_blocks, scar_norm* norm_out, void* workspace, size_t workspace_bytes,
                           void* stream) {
  const uint64_t nb = layout_blocks(layout);
  if (nb == UINT64_MAX) return SCAR_ERR_INVALID_ARG;
  if (tv && layout->dtype != SCAR_F32 && layout->dtype != SCAR_BF16) return SCAR_ERR_UNSUPPORTED;
  const int eb = host_elem_bytes(layout->dtype);
  if (all_blocks) n_idx = (uint32_t)nb;
  if (norm_out) {
    if (!aligned(norm_out, 8)) return SCAR_ERR_INVALID_ARG;
    const int rc = check_workspace(workspace, workspace_bytes, nb);
    if (rc) return rc;
  }
  hipStream_t st = (hipStream_t)stream;
  char* partial = norm_out ? (char*)workspace + kWsNormOffset : nullptr;
  auto finish = [&](uint32_t n_partial) {
    if (tv)
      launch_finish_tv(partial, n_partial, norm_out, st);
    else
      launch_finish(layout->dtype, partial, n_partial, norm_out, st);
  };
  if (n_idx == 0 || nb == 0) {
    if (norm_out) {
      finish(0);
      return launch_status();
    }
    return SCAR_OK;
  }
  if (!x || !c || (!all_blocks && !idx) || !aligned(idx, 4) || !aligned(weights, 4)) return SCAR_ERR_INVALID_ARG;
  if (layout->dtype == SCAR_F32_BF16C)
    return mixed_recover_or_norm(store, packed, layout, (uint32_t)nb, x, c, all_blocks ? nullptr : idx,
                                 n_idx, norm_out, partial, st);
  if (!aligned(x, eb) || !aligned(c, eb)) return SCAR_ERR_INVALID_ARG;
  const bool vec = aligned(x, 16) && aligned(c, 16) && ((uint64_t)layout->block_len * eb) % 16 == 0;
  const uint32_t pieces = row_pieces(layout, eb, vec);
  const int g = pieces > 1 ? 256 : pick_group(layout->block_len, eb, co_aligned(x, c), 1, true);
  const uint32_t n_blocks = (uint32_t)nb;
  // what the pass measures; a recovery without a norm only copies, whatever the metric
  int dt = layout->dtype == SCAR_F32 ? DT_F32 : (layout->dtype == SCAR_BF16 ? DT_BF16 : DT_I32);
  if (tv && norm_out) dt = layout->dtype == SCAR_F32 ? DT_F32_TV : DT_BF16_TV;
  uint32_t n_partial = 0;
  if (!store && norm_out && all_blocks && !packed && !(tv && weights) && aligned(x, 16) && aligned(c, 16)) {
    switch (dt) {  // the whole store, nothing to weigh: no need to look at the blocks
      case DT_F32: n_partial = launch_norm_all<DT_F32>(layout, x, c, partial, st); break;
      case DT_BF16: n_partial = launch_norm_all<DT_BF16>(layout, x, c, partial, st); break;
      case DT_I32: n_partial = launch_norm_all<DT_I32>(layout, x, c, partial, st); break;
      case DT_F32_TV: n_partial = launch_norm_all<DT_F32_TV>(layout, x, c, partial, st); break;
      default: n_partial = launch_norm_all<DT_BF16_TV>(layout, x, c, partial, st); break;
    }
    finish(n_partial);
    return launch_status();
  }
  if (store && norm_out)
    n_partial = dispatch_recover<true, true>(dt, g, layout, x, c, idx, n_idx, n_blocks, pieces, vec, packed, partial, weights, st);
  else if (store)
    dispatch_recover<true, false>(dt, g, layout, x, c, idx, n_idx, n_blocks, pieces, vec, packed, nullptr, nullptr, st);
  else
    n_partial = dispatch_recover<false, true>(dt, g, layout, x, c, idx, n_idx, n_blocks, pieces, vec, packed, partial, weights, st);
  if (norm_out) finish(n_partial);
  return launch_status();
}

}  // namespace scar

using namespace scar;

extern "C" int scar_checkpoint_commit(const scar_layout* layout, const void* x, void* c,
                                      const uint32_t* idx, uint32_t n_idx, void* staging,
                                      void* stream) {
  const uint64_t nb = layout_blocks(layout);
  if (nb == UINT64_MAX) return SCAR_ERR_INVALID_ARG;
  if (n_idx == 0 || nb == 0) return SCAR_OK;
  if (layout->dtype == SCAR_F32_BF16C)
    return mixed_commit(layout, (uint32_t)nb, x, c, idx, n_idx, staging, (hipStream_t)stream);
  const int eb = host_elem_bytes(layout->dtype);
  if (!x || !c || !idx || !aligned(x, eb) || !aligned(c, eb) || !aligned(idx, 4) ||
      (staging && !aligned(staging, eb)))
    return SCAR_ERR_INVALID_ARG;
  const bool row16 = ((uint64_t)layout->block_len * eb) % 16 == 0;
  const bool vec = aligned(x, 16) && aligned(c, 16) && row16;
  const bool vec_st = vec && staging && aligned(staging, 16);
  const uint32_t pieces = row_pieces(layout, eb, vec);
  const int g = pieces > 1 ? 256 : pick_group(layout->block_len, eb, co_aligned(x, c), 1, true);
  hipStream_t st = (hipStream_t)stream;
  if (eb == 4)
    dispatch_commit<uint32_t>(g, layout, x, c, idx, n_idx, staging, (uint32_t)nb, pieces, vec, vec_st, st);
  else
    dispatch_commit<uint16_t>(g, layout, x, c, idx, n_idx, staging, (uint32_t)nb, pieces, vec, vec_st, st);
  return launch_status();
}

extern "C" int scar_partial_recover(const scar_layout* layout, void* x, const void* c,
                                    const uint32_t* lost_idx, uint32_t n_lost, scar_norm* norm_out,
                                    void* workspace, size_t workspace_bytes, void* stream) {
  return recover_or_norm(true, false, false, layout, x, c, nullptr, lost_idx, n_lost, false, norm_out,
                         workspace, workspace_bytes, stream);
}

extern "C" int scar_partial_recover_rows(const scar_layout* layout, void* x, const void* rows,
                                         const uint32_t* lost_idx, uint32_t n_lost, scar_norm* norm_out,
                                         void* workspace, size_t workspace_bytes, void* stream) {
  return recover_or_norm(true, true, false, layout, x, rows, nullptr, lost_idx, n_lost, false, norm_out,
                         workspace, workspace_bytes, stream);
}

extern "C" int scar_perturbation_norm(const scar_layout* layout, const void* x, const void* c,
                                      const uint32_t* idx, uint32_t n_idx, scar_norm* norm_out,
                                      void* workspace, size_t workspace_bytes, void* stream) {
  if (!norm_out) return SCAR_ERR_INVALID_ARG;
  return recover_or_norm(false, false, false, layout, const_cast<void*>(x), c, nullptr, idx, n_idx,
                         idx == nullptr, norm_out, workspace, workspace_bytes, stream);
}

extern "C" int scar_tv_partial_recover(const scar_layout* layout, void* x, const void* c,
                                       const float* weights, const uint32_t* lost_idx, uint32_t n_lost,
                                       scar_norm* norm_out, void* workspace, size_t workspace_bytes,
                                       void* stream) {
  return recover_or_norm(true, false, true, layout, x, c, weights, lost_idx, n_lost, false, norm_out,
                         workspace, workspace_bytes, stream);
}

extern "C" int scar_tv_perturbation_norm(const scar_layout* layout, const void* x, const void* c,
                                         const float* weights, const uint32_t* idx, uint32_t n_idx,
                                         scar_norm* norm_out, void* workspace, size_t workspace_bytes,
                                         void* stream) {
  if (!norm_out) return SCAR_ERR_INVALID_ARG;
  return recover_or_norm(false, false, true, layout, const_cast<void*>(x), c, weights, idx, n_idx,
                         idx == nullptr, norm_out, workspace, workspace_bytes, stream);
}

