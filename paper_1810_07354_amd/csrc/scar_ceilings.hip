// Plain bandwidth kernels: the measured ceilings for the three access shapes of the cycle
// (two-stream read, copy, read-two-write-one).  No index lists, no blocks, next to no
// arithmetic; the access style is that of the path's kernels.
#include "scar_device.hpp"
#include "scar_host.hpp"
#include "../../include/scar_ceilings.h"

namespace scar {

enum : int { CEIL_READ2 = 0, CEIL_COPY = 1, CEIL_READ2_WRITE1 = 2 };

// U 16-byte accesses per lane and stream; each wavefront's U accesses cover one contiguous
// U KiB (as a wavefront of the score scan reads a block).  Measured best per shape on 2 x 4 GiB:
// the read with U = 4 and its workgroups per compute unit limited like the score scan's; the two
// shapes that write with U = 1 and every workgroup used once (a copy with U = 4 is 4 % slower,
// a grid of a few thousand striding workgroups 10-15 % slower).
template <int MODE, int U>
__global__ __launch_bounds__(kWG) void k_ceiling(const uint4* __restrict__ a, uint4* __restrict__ b,
                                                 uint64_t nvec, unsigned long long* __restrict__ sink) {
  uint32_t fold = 0;
  const uint32_t in_wg = (threadIdx.x / kWave) * (U * kWave) + (threadIdx.x & (kWave - 1));
  for (uint64_t v0 = (uint64_t)xcd_contiguous_block_id() * (kWG * U); v0 < nvec;
       v0 += (uint64_t)gridDim.x * (kWG * U)) {
    uint4 av[U], bv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint64_t v = v0 + in_wg + u * kWave;
      av[u] = make_uint4(0, 0, 0, 0), bv[u] = make_uint4(0, 0, 0, 0);
      if (v < nvec) {
        av[u] = load_stream(a + v);
        if (MODE != CEIL_COPY) bv[u] = load_stream(b + v);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint64_t v = v0 + in_wg + u * kWave;
      if (MODE != CEIL_COPY) fold ^= (av[u].x ^ av[u].y ^ av[u].z ^ av[u].w) + (bv[u].x ^ bv[u].y ^ bv[u].z ^ bv[u].w);
      if (MODE != CEIL_READ2 && v < nvec) store_stream(b + v, av[u]);
    }
  }
  if (MODE != CEIL_COPY && fold == 0x9e3779b9u && sink) *sink = fold;  // practically never
}

template <int MODE>
static int launch_ceiling(const void* a, void* b, uint64_t bytes, void* sink, void* stream) {
  if (!a || !b || !aligned(a, 16) || !aligned(b, 16) || bytes % 16 != 0 || (sink && !aligned(sink, 8)))
    return SCAR_ERR_INVALID_ARG;
  if (bytes == 0) return SCAR_OK;
  constexpr int U = MODE == CEIL_READ2 ? kUnroll : 1;
  const uint64_t nvec = bytes / 16;
  const uint64_t need = (nvec + kWG * U - 1) / (kWG * U);
  const uint32_t grid = xcd_grid(need, kScoreGridCap);
  const size_t lds = MODE == CEIL_READ2 ? stream_lds_bytes(need, 2 * 16 * kWG * U) : 0;
  launch((k_ceiling<MODE, U>), dim3(grid), dim3(kWG), lds, (hipStream_t)stream, (const uint4*)a,
         (uint4*)b, nvec, (unsigned long long*)sink);
  return launch_status();
}

}  // namespace scar

using namespace scar;

extern "C" int scar_ceiling_read2(const void* a, const void* b, uint64_t bytes, void* sink, void* stream) {
  return launch_ceiling<CEIL_READ2>(a, const_cast<void*>(b), bytes, sink, stream);
}

extern "C" int scar_ceiling_copy(const void* a, void* b, uint64_t bytes, void* stream) {
  return launch_ceiling<CEIL_COPY>(a, b, bytes, nullptr, stream);
}

extern "C" int scar_ceiling_read2_write1(const void* a, void* b, uint64_t bytes, void* sink, void* stream) {
  return launch_ceiling<CEIL_READ2_WRITE1>(a, b, bytes, sink, stream);
}
