// Host-side helpers shared by the entry points: argument checks, block geometry,
// choice of the group size, and the layout of the caller's workspace.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <tuple>
#include <utility>

#include "../../include/scar.h"

namespace scar {

constexpr uint32_t kMaxBlockLen = 1u << 28;

inline bool dtype_ok(int32_t dt) {
  return dt == SCAR_F32 || dt == SCAR_BF16 || dt == SCAR_I32 || dt == SCAR_F32_BF16C;
}
inline int host_elem_bytes(int32_t dt) { return dt == SCAR_BF16 ? 2 : 4; }  // of x
inline int host_c_elem_bytes(int32_t dt) { return (dt == SCAR_BF16 || dt == SCAR_F32_BF16C) ? 2 : 4; }  // of c

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// n_blocks of a layout, or UINT64_MAX if the layout itself is not acceptable.
inline uint64_t layout_blocks(const scar_layout* l) {
  if (!l || !dtype_ok(l->dtype) || l->block_len == 0 || l->block_len > kMaxBlockLen) return UINT64_MAX;
  const uint64_t nb = l->n_elems / l->block_len + (l->n_elems % l->block_len ? 1 : 0);
  return nb > SCAR_MAX_BLOCKS ? UINT64_MAX : nb;
}

// Group size for blocks of `block_len` elements: the power of two that gives each lane
// about `per_lane` loads per stream (16-byte loads when the streams allow them - by16 -,
// element loads otherwise).  The score kernel reduces inside a group, so it offers {1..64, 256} and
// wants four loads per lane; the row kernels only move data and do best with one
// (measured on 4 KiB rows: 5.66 TB/s with a whole workgroup per row against 5.33 TB/s with
// one wavefront per row), and offer every power of two up to 256.
inline int pick_group_units(uint64_t units, int per_lane, bool allow_128) {
  const uint64_t want = (units + per_lane - 1) / per_lane;
  int g = 1;
  while (g < 256 && (uint64_t)g < want) g <<= 1;
  return (g == 128 && !allow_128) ? 256 : g;
}
inline int pick_group(uint32_t block_len, int ebytes, bool by16, int per_lane, bool allow_128) {
  const uint64_t units = by16 ? ((uint64_t)block_len * ebytes + 15) / 16 : block_len;
  return pick_group_units(units, per_lane, allow_128);
}

// True if a and b sit at the same offset within their 16-byte lines: then rows of the two
// streams can be walked with 16-byte steps between a few leading and trailing elements,
// whatever the row length.
inline bool co_aligned(const void* a, const void* b) {
  return ((reinterpret_cast<uintptr_t>(a) ^ reinterpret_cast<uintptr_t>(b)) & 15) == 0;
}

// ---- workspace layout ---------------------------------------------------------------
// [0, 64 KiB)    selection: digit histograms and pass states        (select)
// [64 KiB, +512 KiB) per-workgroup partial sums of the norm          (recover, norm)
// [576 KiB, ...) per-tile counts of the compaction, 8 bytes per tile (select, mask)
constexpr size_t kWsSelectBytes = 64 * 1024;
constexpr size_t kWsNormOffset = kWsSelectBytes;
constexpr size_t kWsNormBytes = 512 * 1024;
constexpr size_t kWsTileOffset = kWsNormOffset + kWsNormBytes;
constexpr uint32_t kTileKeys = 2048;   // keys per compaction tile
constexpr uint32_t kMaxNormGrid = kWsNormBytes / 8;

constexpr uint64_t n_tiles_of(uint64_t n) { return (n + kTileKeys - 1) / kTileKeys; }

constexpr size_t workspace_bytes_for(uint64_t n_blocks) {
  return kWsTileOffset + ((n_tiles_of(n_blocks) * 8 + 255) / 256) * 256 + 256;
}

inline int check_workspace(const void* ws, size_t bytes, uint64_t n_blocks) {
  if (!ws || !aligned(ws, 256) || bytes < workspace_bytes_for(n_blocks)) return SCAR_ERR_WORKSPACE;
  return SCAR_OK;
}

// Upper bounds on grid sizes; kernels stride over the rest.
constexpr uint64_t kScoreGridCap = 1u << 20;
constexpr uint64_t kCopyGridCap = 1u << 20;

// Grid for `need` workgroups, at most `cap`, rounded up to a multiple of 8 (one share per
// XCD; the kernels skip the overshoot).
inline uint32_t xcd_grid(uint64_t need, uint64_t cap) {
  const uint64_t g = need < cap ? need : cap;
  return (uint32_t)((g + 7) / 8 * 8);
}

// A long streaming read runs fastest with 80-96 KiB of loads in flight per compute unit,
// not with as many workgroups as registers allow: fewer, longer address streams reach the
// memory at a time (2^30 float32 in 1,024-element blocks, 32 KiB in flight per workgroup:
// 1,200 us with eight workgroups per compute unit, 1,160 us with three; 512-element blocks,
// 16 KiB per workgroup: best with four or five).  The streaming kernels use next to no LDS, so
// a launch limits its workgroups per compute unit by asking for LDS it does not use: this
// returns the dynamic LDS bytes for a launch of `grid` workgroups that each keep
// `wg_bytes_in_flight` bytes of loads outstanding (0 = no limit: short launches, and
// workgroups with so little in flight that eight of them are needed anyway).
constexpr uint64_t kStreamFromGrid = 16384;  // half a GiB of loads; below, no gain (6,104 workgroups: 4 % slower)
constexpr uint64_t kStreamBytesPerCu = 86 * 1024;  // 32 KiB a workgroup -> 3, 24 -> 4, 16 -> 5
constexpr size_t kLdsPerCu = 160 * 1024;
inline size_t stream_lds_bytes(uint64_t grid, uint64_t wg_bytes_in_flight) {
  if (grid < kStreamFromGrid || wg_bytes_in_flight == 0) return 0;
  uint64_t wgs = (kStreamBytesPerCu + wg_bytes_in_flight / 2) / wg_bytes_in_flight;
  if (wgs < 3) wgs = 3;
  if (wgs >= 8) return 0;
  return kLdsPerCu / wgs - 1024;
}

// Rows per chunk of the run-of-rows score kernels: as many rows of `row_bytes` bytes as fit
// `max_steps` 16-byte steps, rounded down so that every chunk starts on a 128-byte line, or
// else on the largest power of two down to 16 bytes that the row length allows; 0 if not even
// one such group of rows fits.
inline uint32_t run_chunk_rows(uint64_t row_bytes, uint32_t max_steps) {
  if (row_bytes == 0) return 0;
  const uint64_t fit = (uint64_t)max_steps * 16 / row_bytes;
  for (uint32_t align = 128; align >= 16; align /= 2) {
    uint32_t m = align;  // rows * row_bytes must be a multiple of align
    for (uint64_t v = row_bytes; m > 1 && v % 2 == 0; v /= 2) m /= 2;
    if (fit >= m) return (uint32_t)(fit / m * m);
  }
  return 0;
}

// The copy kernels hand rows longer than kPieceBytes out in pieces of that size (grid y =
// piece).  Grid size in y for rows cut into `pieces`: one slice per piece while
// grid_x * grid_y stays within `cap` workgroups (and the 65,535 of the y dimension); slices
// stride over the rest.
constexpr uint32_t kPieceBytes = 4096;
inline uint32_t piece_grid(uint32_t pieces, uint32_t grid_x, uint64_t cap) {
  uint64_t y = cap / (grid_x ? grid_x : 1);
  if (y > pieces) y = pieces;
  if (y > 65535) y = 65535;
  return y ? (uint32_t)y : 1;
}

// Grid of a row kernel: x over the `need_x` workgroup-sized slots of the index list, y over
// the pieces.  Long lists: x padded to a multiple of 8 (each XCD an eighth of the list, see
// xcd_contiguous_block_id), y as piece_grid says.  A list of fewer than kRowSpreadBelow slots
// whose rows are cut into pieces is spread over the XCDs by its pieces instead (row_grid_slot
// on the device applies the same rule): x is not padded - padding would be idle workgroups,
// seven in eight for a list of one slot - and y is a multiple of 8.
constexpr uint64_t kRowSpreadBelow = 256;
struct RowGrid {
  uint32_t x, y;
};
inline RowGrid row_grid(uint64_t need_x, uint32_t pieces, uint64_t cap) {
  if (pieces > 1 && need_x > 0 && need_x < kRowSpreadBelow) {
    uint64_t y = cap / need_x;
    if (y > pieces) y = pieces;
    if (y > 65528) y = 65528;
    y = y < 8 ? 8 : y / 8 * 8;
    return {(uint32_t)need_x, (uint32_t)y};
  }
  const uint32_t x = xcd_grid(need_x, cap);
  return {x, piece_grid(pieces, x, cap)};
}

// Second stage of the norm (defined with the row kernels): adds n_partial partial sums
// (double, or uint64 for SCAR_I32) in a fixed order and writes *out.
void launch_finish(int32_t dtype, const void* partial, uint32_t n_partial, scar_norm* out,
                   hipStream_t st);
// The same for the scaled total variation: double partial sums of w_b * sum |c - x|; the norm
// is half their sum.
void launch_finish_tv(const void* partial, uint32_t n_partial, scar_norm* out, hipStream_t st);

// ---- reduced-precision checkpoint (SCAR_F32_BF16C: x float32, c bfloat16) ---------------
// Bodies of the entry points for that store type (defined with its kernels); arguments are
// as in the entry points and the layout has already been checked.
bool mixed_giant_scores(const scar_layout* l, uint32_t n_blocks, const void* x, const void* c,
                        const uint32_t* idx, uint32_t n_idx, void* scores, hipStream_t st, int* status);
int mixed_block_scores(const scar_layout* l, uint32_t n_blocks, const void* x, const void* c,
                       const uint32_t* idx, uint32_t n_idx, void* scores, hipStream_t st);
int mixed_commit(const scar_layout* l, uint32_t n_blocks, const void* x, void* c, const uint32_t* idx,
                 uint32_t n_idx, void* staging, hipStream_t st);
int mixed_recover_or_norm(bool store, bool packed, const scar_layout* l, uint32_t n_blocks, void* x, const void* c,
                          const uint32_t* idx, uint32_t n_idx, scar_norm* norm_out, void* partial,
                          hipStream_t st);

// ---- blocks of unequal length ----------------------------------------------------------
// The store is cut into ranges of `range_elems` consecutive elements, one workgroup each; a
// range is a whole number of 4,096-element chunks.  Walks that add something up (scores,
// norms) use at most kVarMaxGrid ranges, because every range hands in a partial sum that a
// single workgroup has to add afterwards; walks that only copy use up to four times as many,
// shorter ones (a 2^30-element store: 16 KiB instead of 64 KiB per workgroup and stream, 800
// -> 744 us on a 4 GB commit).
constexpr uint32_t kVarChunk = 4096;
constexpr uint32_t kVarMaxGrid = 65536;
constexpr uint32_t kVarMaxGridCopy = 4 * kVarMaxGrid;

struct VarGeometry {
  uint64_t range_elems;
  uint32_t n_wg;
};

inline VarGeometry var_geometry(uint64_t n_elems, uint32_t max_grid = kVarMaxGrid) {
  const uint64_t n_chunks = (n_elems + kVarChunk - 1) / kVarChunk;
  uint64_t per = (n_chunks + max_grid - 1) / max_grid;
  if (per == 0) per = 1;
  const uint64_t range = per * kVarChunk;
  return {range, (uint32_t)((n_elems + range - 1) / range)};
}

// Workspace of the variable-length calls: per range its first block (4 bytes) and whether
// it holds a chosen block (1 byte), both sized for the copy walks; then
// 8 * (kVarMaxGrid + n_blocks) bytes of partial sums; then one selection byte per block.
constexpr size_t kVarPlanFirstBytes = 4 * (size_t)kVarMaxGridCopy;
constexpr size_t kVarPlanAnyOffset = kVarPlanFirstBytes;
constexpr size_t kVarPartialOffset = kVarPlanAnyOffset + kVarMaxGridCopy;
inline size_t var_mask_offset(uint64_t n_blocks) {
  return kVarPartialOffset + ((8 * ((size_t)kVarMaxGridCopy + n_blocks) + 255) / 256) * 256;
}
// ... then 8 bytes per block: where the block sits in a packed buffer (staging rows of a
// commit, rows read back from storage).
inline size_t var_pack_offset(uint64_t n_blocks) {
  return var_mask_offset(n_blocks) + ((n_blocks + 255) / 256) * 256;
}
inline size_t var_workspace_bytes_for(uint64_t n_blocks) {
  return var_pack_offset(n_blocks) + ((8 * n_blocks + 255) / 256) * 256 + 256;
}

// ---- enqueueing kernels ---------------------------------------------------------------
// Every kernel goes out through launch(), which keeps the status that HIP returns for that
// very launch: the thread's "last error" state is neither read nor cleared, so a failure
// left behind by the caller's own earlier HIP work is not mistaken for this call's, and
// stays where the caller can still find it.  After a launch has failed, the rest of the
// entry point's launches are skipped; launch_status() ends the entry point: it returns what
// happened and clears the note for the thread's next call.
inline hipError_t& launch_error() {
  static thread_local hipError_t err = hipSuccess;
  return err;
}

template <typename... KArgs, size_t... I>
inline hipError_t launch_packed(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t st,
                                std::tuple<KArgs...>& vals, std::index_sequence<I...>) {
  void* ptrs[sizeof...(KArgs) ? sizeof...(KArgs) : 1] = {(void*)&std::get<I>(vals)...};
  return hipLaunchKernel((const void*)kernel, grid, block, ptrs, lds, st);
}

template <typename... KArgs, typename... Args>
inline void launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t st, Args... args) {
  static_assert(sizeof...(KArgs) == sizeof...(Args), "one argument per kernel parameter");
  if (launch_error() != hipSuccess) return;
  std::tuple<KArgs...> vals{static_cast<KArgs>(args)...};
  launch_error() = launch_packed(kernel, grid, block, lds, st, vals, std::index_sequence_for<KArgs...>{});
}

inline int launch_status() {
  const hipError_t err = launch_error();
  launch_error() = hipSuccess;
  return err == hipSuccess ? SCAR_OK : SCAR_ERR_DEVICE;
}

}  // namespace scar
