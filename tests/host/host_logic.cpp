// Host-side launch arithmetic of the library, checked without a GPU: no HIP call is made.
// Built and run by tests/test_host_logic.py.
#include <cstdio>
#include <cstdlib>

#include "../../paper_1810_07354_amd/csrc/scar_host.hpp"

using namespace scar;

static int failures = 0;
#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) {                                                         \
      std::printf("FAILED line %d: %s\n", __LINE__, #cond);                \
      ++failures;                                                          \
    }                                                                      \
  } while (0)

int main() {
  // grids: a multiple of 8 (one share per XCD), never above the cap rounded up
  for (uint64_t need : {0ull, 1ull, 7ull, 8ull, 9ull, 1000ull, (1ull << 20) - 3, 1ull << 20, 1ull << 30}) {
    const uint32_t g = xcd_grid(need, kScoreGridCap);
    CHECK(g % 8 == 0);
    CHECK(g >= (need < kScoreGridCap ? need : kScoreGridCap));
    CHECK(g <= ((kScoreGridCap + 7) / 8) * 8);
  }
  // group sizes: a power of two that gives each lane at most `per_lane` units, 128 only on request
  for (uint64_t units = 1; units <= 5000; units += (units < 300 ? 1 : 97)) {
    for (int per_lane : {1, 2, 4}) {
      const int g = pick_group_units(units, per_lane, false), g128 = pick_group_units(units, per_lane, true);
      CHECK((g & (g - 1)) == 0 && g >= 1 && g <= 256 && g != 128);
      CHECK((g128 & (g128 - 1)) == 0 && g128 <= 256);
      if (g < 256) CHECK((uint64_t)g * per_lane >= units);
      if (g > 1 && g != 256) CHECK((uint64_t)(g / 2) * per_lane < units);
    }
  }
  // pieces: grid_x * grid_y within the cap, y within the pieces and the launch limit
  for (uint32_t pieces : {1u, 2u, 17u, 4096u, 100000u})
    for (uint32_t gx : {8u, 1024u, 65536u}) {
      const uint32_t gy = piece_grid(pieces, gx, kMaxNormGrid);
      CHECK(gy >= 1 && gy <= pieces && gy <= 65535);
      CHECK(gy == 1 || (uint64_t)gx * gy <= kMaxNormGrid);
    }
  // grids of the row kernels: long lists pad x to the XCDs and keep x * y within the cap; a
  // short list of rows in pieces is not padded in x, has a y that is a multiple of 8 (the
  // device renumbers the whole grid in eighths) and still stays within the cap
  for (uint64_t cap : {(uint64_t)kMaxNormGrid, kCopyGridCap})
    for (uint32_t pieces : {1u, 2u, 5u, 8u, 17u, 4096u, 65536u, 100000u})
      for (uint64_t need : {1ull, 2ull, 7ull, 100ull, 255ull, 256ull, 5000ull, 1ull << 20}) {
        const RowGrid rg = row_grid(need, pieces, cap);
        CHECK(rg.x >= 1 && rg.y >= 1 && rg.y <= 65535);
        if (pieces > 1 && need < kRowSpreadBelow) {
          CHECK(rg.x == need && rg.y % 8 == 0);
          CHECK((uint64_t)rg.x * rg.y <= cap);
          CHECK(rg.y <= (pieces + 7) / 8 * 8);
        } else {
          CHECK(rg.x % 8 == 0 && rg.y <= pieces);
          CHECK(rg.y == 1 || (uint64_t)rg.x * rg.y <= cap);
        }
      }
  // workgroups per compute unit of the streaming reads: none asked for on short launches or
  // when eight fit anyway; otherwise exactly the wanted number fits the 160 KiB
  CHECK(stream_lds_bytes(kStreamFromGrid - 1, 32 * 1024) == 0);
  CHECK(stream_lds_bytes(1 << 20, 0) == 0);
  CHECK(stream_lds_bytes(1 << 20, 8 * 1024) == 0);
  struct { uint64_t in_flight; unsigned want; } cases[] = {{32 * 1024, 3}, {24 * 1024, 4}, {16 * 1024, 5}, {64 * 1024, 3}};
  for (auto cs : cases) {
    const size_t lds = stream_lds_bytes(1 << 20, cs.in_flight);
    CHECK(lds > 0 && lds <= 64 * 1024);
    CHECK(cs.want * (lds + 64) <= kLdsPerCu);        // that many fit (with a little static LDS)
    CHECK((cs.want + 1) * lds > kLdsPerCu);          // one more does not
  }
  // chunks of the run-of-rows kernels: whole rows, within the step budget, starting on a
  // 16-byte boundary at least and on a 128-byte line whenever some row count allows it
  for (uint32_t max_steps : {1024u}) {
    for (uint64_t rb = 2; rb <= 4200; rb += 2) {      // elements are 2 or 4 bytes: rows are even
      const uint32_t rows = run_chunk_rows(rb, max_steps);
      if (rb <= 2048) CHECK(rows > 0);               // 8 rows of 2 KiB always fit
      if (rows == 0) continue;
      CHECK(rows * rb <= (uint64_t)max_steps * 16);
      CHECK(rows * rb % 16 == 0);
      uint64_t m128 = 128;                           // rows needed for a whole number of lines
      for (uint64_t v = rb; m128 > 1 && v % 2 == 0; v /= 2) m128 /= 2;
      if (m128 * rb <= (uint64_t)max_steps * 16) CHECK(rows * rb % 128 == 0);
      CHECK(rows + m128 > (uint64_t)max_steps * 16 / rb || rows * rb % 128 != 0);  // as many as fit
    }
  }
  CHECK(run_chunk_rows(0, 1024) == 0);
  CHECK(run_chunk_rows(4090, 1024) == 0);            // 8 rows would be needed, 4 fit
  CHECK(run_chunk_rows(400, 1024) == 40);            // 40 rows = 125 lines
  // layout checks
  scar_layout l = {SCAR_F32, 1024, (1ull << 30)};
  CHECK(layout_blocks(&l) == (1u << 20));
  l.n_elems += 1;
  CHECK(layout_blocks(&l) == (1u << 20) + 1);
  l.block_len = 0;
  CHECK(layout_blocks(&l) == UINT64_MAX);
  CHECK(workspace_bytes_for(1 << 20) >= kWsTileOffset + (1 << 20) / kTileKeys * 8);
  if (failures == 0) std::printf("host logic ok\n");
  return failures ? 1 : 0;
}
