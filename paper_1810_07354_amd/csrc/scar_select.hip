// scar_select_topk: the k blocks with the largest scores (checkpoint step 3 of
// Section 4.3), and scar_mask_to_indices.
//
// Scores become unsigned keys whose integer order is the score order (NaN on top, -0
// equal to +0).  A most-significant-digit-first radix select finds the k-th largest key
// T: each pass builds a histogram of one digit of the keys that still match the prefix
// found so far (LDS histogram per workgroup, then one global atomic per non-empty bin).
// The next kernel in the stream walks the finished histogram from the top and fixes the
// digit - every workgroup does this small walk for itself, so no workgroup ever waits
// for another and no device-wide fence is needed inside a kernel.
// After the last pass every key > T is selected together with the first `take` keys
// equal to T in index order, where take = k - #(keys > T).
//
// The chosen indices are then written in ascending order by one kernel: every workgroup
// classifies one tile of 2,048 keys, publishes its counts and looks back over the tiles
// before it for the sum of theirs (a chained scan), so the result does not depend on the
// order in which workgroups run.
#include <mutex>

#include "scar_device.hpp"
#include "scar_host.hpp"

namespace scar {

constexpr int kMaxBins = 2048;
constexpr int kMaxPasses = 6;
constexpr int kKeysPerThread = kTileKeys / kWG;  // 8 consecutive keys per thread
// A histogram pass reads its keys from wherever the score kernel left them (usually another
// XCD's L2 or HBM), so many small tiles - many loads in flight - beat few large ones, although
// larger tiles would save global atomics at the end of the pass (measured both ways).
constexpr int kHistKeysPerThread = kKeysPerThread;
constexpr uint32_t kHistTileKeys = kHistKeysPerThread * kWG;

enum : int { SRC_F32 = 0, SRC_I64 = 1, SRC_MASK = 2, SRC_RANDOM = 3 };

// Where the keys come from: an array in device memory, or (SRC_RANDOM) the counter-based
// generator, which needs no memory at all.
struct KeyArgs {
  const void* ptr;
  uint64_t seed;
  uint64_t draw;
  // 64-bit integer scores: number of 11-bit digits (6 covers all 64 bits) and, when `bounded`,
  // the largest score the caller vouches for - scores are then clamped into [0, cap], whose
  // keys fit `passes` digits
  int passes;
  int bounded;
  unsigned long long cap;
};

inline KeyArgs key_args(const void* ptr, uint64_t seed = 0, uint64_t draw = 0) {
  return KeyArgs{ptr, seed, draw, 6, 0, ~0ull};
}

// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, "Parallel random numbers: as easy as 1, 2,
// 3", SC'11), first output word: ten rounds of
//   (c0,c1,c2,c3) <- (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1, lo(M0*c0)),
// the key stepping by (W0, W1) between rounds.
__device__ __forceinline__ uint32_t philox4x32_10_word0(uint32_t c0, uint32_t c1, uint32_t c2,
                                                        uint32_t c3, uint32_t k0, uint32_t k1) {
  constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t h0 = __umulhi(M0, c0), l0 = M0 * c0;
    const uint32_t h1 = __umulhi(M1, c2), l1 = M1 * c2;
    c0 = h1 ^ c1 ^ k0;
    c1 = l1;
    c2 = h0 ^ c3 ^ k1;
    c3 = l0;
    k0 += W0;
    k1 += W1;
  }
  return c0;
}

struct SelectState {
  unsigned long long prefix;  // digits fixed so far, right-aligned
  uint32_t k_rem;             // how many of the keys matching `prefix` are still to be taken
  uint32_t pad;
};

// Layout of the selection part of the workspace.  state[p] is the state before pass p.
struct SelectWs {
  uint32_t hist[kMaxPasses][kMaxBins];
  SelectState state[kMaxPasses + 1];
};
static_assert(sizeof(SelectWs) <= kWsSelectBytes, "selection scratch exceeds its share");

template <int SRC>
struct Key;

template <>
struct Key<SRC_F32> {
  using type = uint32_t;
  __host__ __device__ static int passes(const KeyArgs&) { return 3; }
  __device__ static int shift(const KeyArgs&, int p) { return p == 0 ? 21 : (p == 1 ? 10 : 0); }
  __device__ static int bits(const KeyArgs&, int p) { return p == 2 ? 10 : 11; }
  __device__ static type load(const KeyArgs& a, uint64_t i) {
    uint32_t u = __float_as_uint(((const float*)a.ptr)[i]);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0xffffffffu;  // NaN: above everything
    if (u == 0x80000000u) u = 0;                              // -0 == +0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  }
};

// 64-bit integer scores: `passes` digits of 11 bits, the last one at bit 0.  Six digits cover
// every int64 (the first then holds the top 9 bits); a caller who knows an upper bound of
// the scores gets fewer (scar_select_topk_bounded): the digits above the bound are the same
// in every key, and a pass that can only find that out is a launch saved.
template <>
struct Key<SRC_I64> {
  using type = unsigned long long;
  __host__ __device__ static int passes(const KeyArgs& a) { return a.passes; }
  __device__ static int shift(const KeyArgs& a, int p) { return 11 * (a.passes - 1 - p); }
  __device__ static int bits(const KeyArgs&, int) { return 11; }
  __device__ static type load(const KeyArgs& a, uint64_t i) {
    const long long v = ((const long long*)a.ptr)[i];
    if (a.bounded) {
      const unsigned long long u = v < 0 ? 0ull : (unsigned long long)v;
      return u > a.cap ? a.cap : u;
    }
    return (unsigned long long)v ^ 0x8000000000000000ull;
  }
};

// The "random" strategy of Section 5.4: block i draws the 32-bit number
// Philox4x32-10(counter = (i, 0, draw), key = seed)[0]; the k largest numbers win.
template <>
struct Key<SRC_RANDOM> {
  using type = uint32_t;
  __host__ __device__ static int passes(const KeyArgs&) { return 3; }
  __device__ static int shift(const KeyArgs&, int p) { return p == 0 ? 21 : (p == 1 ? 10 : 0); }
  __device__ static int bits(const KeyArgs&, int p) { return p == 2 ? 10 : 11; }
  __device__ static type load(const KeyArgs& a, uint64_t i) {
    return philox4x32_10_word0((uint32_t)i, 0u, (uint32_t)a.draw, (uint32_t)(a.draw >> 32),
                               (uint32_t)a.seed, (uint32_t)(a.seed >> 32));
  }
};

template <>
struct Key<SRC_MASK> {  // only classified, never histogrammed
  using type = uint32_t;
  __host__ __device__ static int passes(const KeyArgs&) { return 0; }
  __device__ static type load(const KeyArgs& a, uint64_t i) { return ((const uint8_t*)a.ptr)[i] ? 1u : 0u; }
};

// Zeroes the histograms and the per-tile words of the compaction, and sets the state before
// the first pass.  `ws_words`: 32-bit words of the selection scratch to clear.
__global__ __launch_bounds__(kWG) void k_select_clear(SelectWs* ws, uint32_t ws_words, uint32_t k,
                                                      unsigned long long* __restrict__ tile_state,
                                                      uint32_t n_tiles) {
  uint32_t* words = (uint32_t*)ws;
  const uint32_t tid = blockIdx.x * kWG + threadIdx.x, nthreads = gridDim.x * kWG;
  for (uint32_t i = tid; i < ws_words; i += nthreads)
    words[i] = (i == offsetof(SelectWs, state[0].k_rem) / 4) ? k : 0u;
  for (uint32_t t = tid; t < n_tiles; t += nthreads) tile_state[t] = 0ull;
}

// Given the finished histogram of one digit and the state before that digit, walk the
// bins from the top down to the one that holds the k_rem-th largest remaining key.
// Every thread of the workgroup (NT threads) gets the state after the digit.  `scratch` is
// LDS for NT / kWave + 1 counters, `result` LDS for one state.
template <int NT = kWG>
__device__ __forceinline__ SelectState next_state(const uint32_t* __restrict__ gh, int bits,
                                                  const SelectState cur, uint32_t* scratch,
                                                  SelectState* result) {
  const int nbins = 1 << bits;
  constexpr int kOwn = kMaxBins / NT;  // thread t owns bins nbins-1-kOwn*t ... nbins-kOwn-kOwn*t
  uint32_t own[kOwn];
  uint32_t cnt = 0;
#pragma unroll
  for (int j = 0; j < kOwn; ++j) {
    const int b = nbins - 1 - ((int)threadIdx.x * kOwn + j);
    own[j] = b >= 0 ? gh[b] : 0;
    cnt += own[j];
  }
  uint32_t total;
  uint32_t above = workgroup_exclusive_scan<NT>(cnt, scratch, &total);
  if (above < cur.k_rem && cur.k_rem <= above + cnt) {  // true in exactly one thread
#pragma unroll
    for (int j = 0; j < kOwn; ++j) {
      if (above + own[j] >= cur.k_rem) {
        const int b = nbins - 1 - ((int)threadIdx.x * kOwn + j);
        result->prefix = (cur.prefix << bits) | (unsigned long long)b;
        result->k_rem = cur.k_rem - above;
        result->pad = 0;
        break;
      }
      above += own[j];
    }
  }
  __syncthreads();
  return *result;
}

// One radix pass over tiles of kTileKeys keys.  Each workgroup first derives the state
// before this pass from the previous pass's finished histogram (all workgroups compute
// the same values; workgroup 0 also stores them for later kernels), then adds the digit
// histogram of the keys that match the prefix.
template <int SRC>
__global__ __launch_bounds__(kWG) void k_select_hist(const KeyArgs scores, uint32_t n,
                                                     uint32_t n_tiles, int pass,
                                                     SelectWs* __restrict__ ws) {
  using K = Key<SRC>;
  using key_t = typename K::type;
  __shared__ uint32_t lh[kMaxBins];
  __shared__ uint32_t scratch[kWG / kWave + 1];
  __shared__ SelectState shared_state;
  for (int b = threadIdx.x; b < kMaxBins; b += kWG) lh[b] = 0;
  // The keys of the first tile are requested before the small histogram walk below, so
  // that their latency (the scores usually sit in another XCD's L2) overlaps with it.
  auto load_tile = [&](uint32_t tile, key_t (&key)[kHistKeysPerThread]) {
    const uint64_t base = (uint64_t)tile * kHistTileKeys + threadIdx.x;
#pragma unroll
    for (int j = 0; j < kHistKeysPerThread; ++j) {
      const uint64_t i = base + (uint64_t)j * kWG;
      key[j] = K::load(scores, i < n ? i : n - 1);
    }
  };
  key_t key[kHistKeysPerThread];
  uint32_t tile = blockIdx.x;
  if (tile < n_tiles) load_tile(tile, key);
  SelectState cur = ws->state[pass == 0 ? 0 : pass - 1];
  if (pass > 0) {
    cur = next_state(ws->hist[pass - 1], K::bits(scores, pass - 1), cur, scratch, &shared_state);
    if (blockIdx.x == 0 && threadIdx.x == 0) ws->state[pass] = cur;
  }
  __syncthreads();
  const int shift = K::shift(scores, pass), bits = K::bits(scores, pass);
  const uint32_t mask = (1u << bits) - 1;
  while (tile < n_tiles) {
    const uint64_t base = (uint64_t)tile * kHistTileKeys + threadIdx.x;
#pragma unroll
    for (int j = 0; j < kHistKeysPerThread; ++j) {
      const uint64_t i = base + (uint64_t)j * kWG;
      const bool match = pass == 0 || (key[j] >> (shift + bits)) == (key_t)cur.prefix;
      const bool on = i < n && match;
      const uint32_t bin = (uint32_t)(key[j] >> shift) & mask;
      if constexpr (SRC == SRC_I64) {
        // the top digits of small integer scores are all alike: a wavefront whose keys fall
        // into one bin adds its count once instead of 64 adds to the same LDS word in a row
        const unsigned long long act = __ballot(on);
        if (act) {
          const int leader = __ffsll((long long)act) - 1;
          const uint32_t bin0 = __shfl(bin, leader, kWave);
          if (__ballot(on && bin == bin0) == act) {
            if ((int)(threadIdx.x & (kWave - 1)) == leader) atomicAdd(&lh[bin0], (uint32_t)__popcll(act));
          } else if (on) {
            atomicAdd(&lh[bin], 1u);
          }
        }
      } else {
        if (on) atomicAdd(&lh[bin], 1u);
      }
    }
    tile += gridDim.x;
    if (tile < n_tiles) load_tile(tile, key);
  }
  __syncthreads();
  uint32_t* gh = ws->hist[pass];
  for (int b = threadIdx.x; b < kMaxBins; b += kWG)
    if (lh[b]) atomicAdd(&gh[b], lh[b]);
}

// ---- ordered compaction in one kernel ---------------------------------------------------
// Workgroup t classifies tile t of kTileKeys keys (a span of consecutive tiles when there are
// more tiles than kCompactMaxGroups; "tile" below then reads "span"), counts its keys above and
// equal to the threshold, publishes the counts in the tile's 64-bit word and adds up the words
// of the tiles before it, a workgroup's width at a time, until it meets a tile that already
// knows its own running total (a chained scan with look-back).  A word carries its own validity:
// bits 63-62 say what it holds (0 nothing yet, 1 the tile's own counts, 2 the running total up
// to and including the tile), bits 61-31 the keys equal to the threshold, bits 30-0 the keys
// above it.  It is written and read with single relaxed device-scope atomic accesses; nothing
// else has to be ordered, so there is no fence.  The words are zeroed by k_select_clear.
//
// A workgroup only ever waits for tiles with lower numbers, and the hardware starts the
// workgroups of a grid in the order of their numbers (per XCD), so the tiles waited for are
// running or done.  (Handing tiles out by a ticket - one atomic counter - would not depend on
// that order, but 512 adds to one address cost 8 us on 2^20 keys.)  The kernel's end does not
// depend on it either: the wait is bounded.  After `spin_limit` polls a workgroup stops
// waiting and counts the keys of all earlier tiles itself - slow, but it always ends, and the
// result is the same.
constexpr unsigned long long kTileOwn = 1ull << 62, kTileRunning = 2ull << 62, kTileFlags = 3ull << 62;
constexpr unsigned long long kTilePayload = ~kTileFlags;
constexpr int kEqualShift = 31;
constexpr uint32_t kFieldMask = 0x7fffffffu;

__device__ __forceinline__ unsigned long long tile_word_load(const unsigned long long* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void tile_word_store(unsigned long long* p, unsigned long long v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <typename T>
__device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
  for (int m = kWave / 2; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
  return v;
}

// Called by the whole workgroup: publishes `own` (the payload of tile `tile`) and returns the
// summed payloads of tiles 0 .. tile-1 in every thread.  Each of the four wavefronts polls 64
// of the 256 tiles of a window; the nearest tile with a running total ends the walk.
// *gave_up (LDS) is set if a predecessor's word did not appear within spin_limit polls (the
// return value is then void).  `part`, `found`: LDS for one value per wavefront.
__device__ __forceinline__ unsigned long long look_back(unsigned long long* __restrict__ tile_state,
                                                        uint32_t tile, unsigned long long own,
                                                        uint32_t spin_limit, int* gave_up,
                                                        unsigned long long* part, int* found) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  if (threadIdx.x == 0) {
    *gave_up = 0;
    tile_word_store(&tile_state[tile], (tile == 0 ? kTileRunning : kTileOwn) | own);
  }
  __syncthreads();
  if (tile == 0) return 0;
  unsigned long long running = 0;
  long long top = (long long)tile - 1;  // highest tile of the window still to be added
  for (;;) {
    const long long t = top - wave * kWave - lane;
    unsigned long long w;
    uint32_t polls = 0;
    bool timed_out = false;
    for (;;) {
      // tiles before the first count as a running total of nothing
      w = t >= 0 ? tile_word_load(&tile_state[t]) : kTileRunning;
      if (__ballot((w & kTileFlags) == 0) == 0) break;
      if (++polls > spin_limit) {
        timed_out = true;
        break;
      }
      __builtin_amdgcn_s_sleep(1);
    }
    const unsigned long long has_total = __ballot((w & kTileFlags) == kTileRunning);
    const int first = has_total ? __ffsll((long long)has_total) - 1 : kWave;
    const unsigned long long sum = wave_sum(lane <= first ? (w & kTilePayload) : 0ull);
    if (lane == 0) {
      part[wave] = sum;
      found[wave] = has_total != 0;
      if (timed_out) *gave_up = 1;
    }
    __syncthreads();
    bool done = false;
    unsigned long long add = 0;
#pragma unroll
    for (int v = 0; v < kWG / kWave; ++v) {
      if (!done) add += part[v];
      done = done || found[v];
    }
    const int stop = *gave_up;
    __syncthreads();  // the slots are rewritten in the next round
    if (stop) return 0;
    running += add;
    if (done) break;
    top -= kWG;
  }
  if (threadIdx.x == 0) tile_word_store(&tile_state[tile], kTileRunning | (running + own));
  return running;
}

// Writes the selected indices at their final, ascending positions.  For a selection the
// threshold is first derived from the last pass's histogram, as in k_select_hist.  out_count
// (mask compaction): receives the number of indices written.
//
// Workgroup w owns the `span` consecutive tiles from w * span on and word w of tile_state; grid =
// ceil(n_tiles / span).  span = 1 (up to kCompactMaxGroups tiles): the tile's keys are
// classified once and stay in registers across the look-back.  Longer key arrays would put
// more tiles in flight than a look-back can cross quickly - every workgroup would walk back
// over all the tiles that run beside it, a window and a round trip across the chip at a time
// (67 M keys: 435 us, a seventh of what the memory allows) - so there a workgroup first counts
// all the keys of its span, publishes one word, adds up the words of the at most
// kCompactMaxGroups - 1 workgroups before it, all of which count at the same time, and then
// places its keys: those of the first kCompactKeptTiles tiles from the classes it kept in LDS while
// counting (two bits per key), those of further tiles (beyond 134 M keys) by reading them again.
constexpr uint32_t kCompactMaxGroups = 2048;
constexpr uint32_t kCompactKeptTiles = 32;  // tiles of a span whose classes wait in LDS (16 KiB)

__device__ __forceinline__ unsigned long long pack_counts(uint32_t above_equal16) {
  return (unsigned long long)(above_equal16 & 0xffffu) | ((unsigned long long)(above_equal16 >> 16) << kEqualShift);
}

template <int SRC>
__global__ __launch_bounds__(kWG) void k_compact(const KeyArgs src, uint32_t n, uint32_t n_tiles, uint32_t span,
                                                 int passes, SelectWs* __restrict__ ws,
                                                 unsigned long long* __restrict__ tile_state,
                                                 uint32_t* __restrict__ out_idx, uint32_t out_cap,
                                                 uint32_t* __restrict__ out_count, uint32_t spin_limit) {
  using key_t = typename Key<SRC>::type;
  constexpr int kWaves = kWG / kWave;
  __shared__ uint32_t slots[kWaves + 1];
  __shared__ unsigned long long wide[kWaves];
  __shared__ SelectState shared_state;
  __shared__ unsigned long long s_before;
  __shared__ int s_gave_up;
  __shared__ int s_found[kWaves];
  __shared__ uint32_t wave_cnt[kKeysPerThread][kWaves];
  __shared__ uint16_t codes[kCompactKeptTiles][kWG];
  key_t T = 0;
  uint32_t take = 0;
  if constexpr (SRC != SRC_MASK) {
    const SelectState fin = next_state(ws->hist[passes - 1], Key<SRC>::bits(src, passes - 1),
                                       ws->state[passes - 1], slots, &shared_state);
    T = (key_t)fin.prefix;
    take = fin.k_rem;
  }
  const uint32_t group = blockIdx.x;
  const uint64_t first64 = (uint64_t)group * span;
  if (first64 >= n_tiles) return;  // cannot happen with the grid above; keeps every access in range
  const uint32_t first = (uint32_t)first64;
  const uint32_t last = n_tiles - first < span ? n_tiles : first + span;  // one past the span's last tile
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const unsigned long long below = (1ull << lane) - 1;  // the lanes before this one

  // A tile is read as kKeysPerThread rows of kWG consecutive keys, thread i taking key i of every
  // row: coalesced, and in index order when rows are taken one after the other and threads in
  // order.  Counts are kept in pairs: low half above the threshold, high half equal to it (a
  // tile holds 2,048 keys).  Key j of this thread in tile t:
  auto key_index = [&](uint32_t t, int j) { return (uint64_t)t * kTileKeys + (uint32_t)j * kWG + threadIdx.x; };
  auto load_tile = [&](uint32_t t, key_t (&key)[kKeysPerThread]) {
#pragma unroll
    for (int j = 0; j < kKeysPerThread; ++j) {
      const uint64_t i = key_index(t, j);
      key[j] = Key<SRC>::load(src, i < n ? i : n - 1);
    }
  };
  // 0 = not selected on its own, 1 = above the threshold, 2 = equal to it
  auto class_of = [&](key_t key, uint64_t i) {
    if (i >= n) return 0;
    if constexpr (SRC == SRC_MASK) return key ? 1 : 0;
    return key > T ? 1 : (key == T ? 2 : 0);
  };
  // This thread's share of the counts of tile t; *code gets the classes of its keys, two bits each.
  auto count_tile = [&](uint32_t t, uint16_t* code) {
    key_t key[kKeysPerThread];
    load_tile(t, key);
    uint32_t cnt = 0, packed = 0;
#pragma unroll
    for (int j = 0; j < kKeysPerThread; ++j) {
      const int c = class_of(key[j], key_index(t, j));
      cnt += c == 1 ? 1u : (c == 2 ? (1u << 16) : 0u);
      packed |= (uint32_t)c << (2 * j);
    }
    *code = (uint16_t)packed;
    return cnt;
  };
  // cls: classes of this thread's keys of a tile.  rank_tile returns the counts of the whole tile
  // and leaves in before_in_tile[j] the counts of everything in the tile that precedes key j of
  // this thread.
  int cls[kKeysPerThread];
  uint32_t before_in_tile[kKeysPerThread];
  auto rank_tile = [&]() {  // from cls[]
    __syncthreads();  // wave_cnt may still be read from the tile before
#pragma unroll
    for (int j = 0; j < kKeysPerThread; ++j) {
      const unsigned long long above = __ballot(cls[j] == 1), equal = __ballot(cls[j] == 2);
      before_in_tile[j] = (uint32_t)__popcll(above & below) | ((uint32_t)__popcll(equal & below) << 16);
      if (lane == 0) wave_cnt[j][wave] = (uint32_t)__popcll(above) | ((uint32_t)__popcll(equal) << 16);
    }
    __syncthreads();
    uint32_t running = 0;
#pragma unroll
    for (int j = 0; j < kKeysPerThread; ++j) {
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        if (w == wave) before_in_tile[j] += running;
        running += wave_cnt[j][w];
      }
    }
    return running;
  };

  auto classes_from_keys = [&](uint32_t t, const key_t (&key)[kKeysPerThread]) {
#pragma unroll
    for (int j = 0; j < kKeysPerThread; ++j) cls[j] = class_of(key[j], key_index(t, j));
  };
  uint32_t total = 0;
  unsigned long long own;
  key_t cur[kKeysPerThread] = {}, nxt[kKeysPerThread] = {};
  const uint32_t kept = last - first < kCompactKeptTiles ? last - first : kCompactKeptTiles;  // tiles with codes in LDS
  if (span == 1) {
    load_tile(first, cur);
    classes_from_keys(first, cur);
    total = rank_tile();
    own = pack_counts(total);
  } else {
    unsigned long long mine = 0;
#pragma unroll 2
    for (uint32_t t = first; t < last; ++t) {
      uint16_t code;
      mine += pack_counts(count_tile(t, &code));
      if (t - first < kCompactKeptTiles) codes[t - first][threadIdx.x] = code;  // read back by the same thread
    }
    own = workgroup_sum(mine, wide);
    if (first + kept < last) load_tile(first + kept, cur);  // on its way during the look-back
  }
  unsigned long long before = look_back(tile_state, group, own, spin_limit, &s_gave_up, wide, s_found);
  if (s_gave_up) {  // count the keys of the earlier tiles directly
    unsigned long long c2 = 0;
    for (uint32_t t = 0; t < first; ++t) {
      uint16_t code;
      c2 += pack_counts(count_tile(t, &code));
    }
    before = workgroup_sum(c2, wide);
    __syncthreads();
    if (threadIdx.x == 0) {
      s_before = before;
      tile_word_store(&tile_state[group], kTileRunning | (before + own));  // later workgroups may stop here
    }
    __syncthreads();
    before = s_before;
  }
  for (uint32_t t = first; t < last; ++t) {
    if (span != 1) {
      if (t - first < kept) {  // classes kept from the count
        const uint32_t code = codes[t - first][threadIdx.x];
#pragma unroll
        for (int j = 0; j < kKeysPerThread; ++j) cls[j] = (int)((code >> (2 * j)) & 3u);
      } else {  // read again, the next tile's keys asked for before this tile is placed
        if (t + 1 < last) load_tile(t + 1, nxt);
        classes_from_keys(t, cur);
      }
      total = rank_tile();
    }
    const uint32_t above0 = (uint32_t)(before & kFieldMask), equal0 = (uint32_t)((before >> kEqualShift) & kFieldMask);
#pragma unroll
    for (int j = 0; j < kKeysPerThread; ++j) {
      const uint32_t n_above = above0 + (before_in_tile[j] & 0xffffu), n_equal = equal0 + (before_in_tile[j] >> 16);
      if (cls[j] == 1) {
        const uint32_t pos = n_above + (n_equal < take ? n_equal : take);
        if (pos < out_cap) out_idx[pos] = (uint32_t)key_index(t, j);
      } else if (cls[j] == 2 && n_equal < take) {
        const uint32_t pos = n_above + n_equal;
        if (pos < out_cap) out_idx[pos] = (uint32_t)key_index(t, j);
      }
    }
    before += pack_counts(total);
    if (t - first >= kept) {
#pragma unroll
      for (int j = 0; j < kKeysPerThread; ++j) cur[j] = nxt[j];
    }
  }
  if (out_count && last == n_tiles && threadIdx.x == 0) *out_count = (uint32_t)(before & kFieldMask);
}

// Whole selection in one workgroup of 1,024 threads for small stores (n <= kSmallSelect):
// keys stay in registers (up to KPT consecutive keys per thread, KPT = 8 or 16 by n),
// histograms in LDS, one launch instead of six or nine.  Its time grows with n (12 us at
// 8,192 float keys, 19 us at 16,384, 35 us at 32,768) while the tiled passes below stay near
// 25 us (40 us for 64-bit keys) up to a few hundred thousand keys, hence the limit.
constexpr int kSmallWG = 1024;
constexpr uint32_t kSmallSelect = 16 * kSmallWG;
template <int SRC, int KPT>
__global__ __launch_bounds__(kSmallWG) void k_select_small(const KeyArgs scores, uint32_t n,
                                                           uint32_t k, uint32_t* __restrict__ out_idx) {
  using K = Key<SRC>;
  using key_t = typename K::type;
  constexpr int kSmallKeys = KPT;
  __shared__ uint32_t lh[kMaxBins];
  __shared__ uint32_t scratch[kSmallWG / kWave + 1];
  __shared__ SelectState shared_state;
  // thread t holds the kpt consecutive keys from t * kpt on (kpt = ceil(n / 1024) <= KPT), so
  // every thread has work whatever n is, and index order is thread order
  const uint32_t kpt = (n + kSmallWG - 1) / kSmallWG;
  const uint32_t base = threadIdx.x * kpt;
  key_t key[kSmallKeys];
#pragma unroll
  for (int j = 0; j < kSmallKeys; ++j)
    key[j] = (uint32_t)j < kpt ? K::load(scores, base + j < n ? base + j : n - 1) : (key_t)0;

  SelectState cur;
  cur.prefix = 0, cur.k_rem = k, cur.pad = 0;
  const int n_passes = K::passes(scores);
  for (int pass = 0; pass < n_passes; ++pass) {
    for (int b = threadIdx.x; b < kMaxBins; b += kSmallWG) lh[b] = 0;
    __syncthreads();
    const int shift = K::shift(scores, pass), bits = K::bits(scores, pass);
    const uint32_t mask = (1u << bits) - 1;
#pragma unroll
    for (int j = 0; j < kSmallKeys; ++j) {
      const bool match = pass == 0 || (key[j] >> (shift + bits)) == (key_t)cur.prefix;
      const bool on = (uint32_t)j < kpt && base + j < n && match;
      const uint32_t bin = (uint32_t)(key[j] >> shift) & mask;
      // When a whole wavefront hits one bin (the top digits of small integer scores are all
      // alike) its 64 adds to one LDS word would run one after the other: add the count once.
      // (64-bit integer keys only: float scores rarely agree, and the test costs them 1-2 us.)
      if constexpr (SRC == SRC_I64) {
        const unsigned long long act = __ballot(on);
        if (act) {
          const int leader = __ffsll((long long)act) - 1;
          const uint32_t bin0 = __shfl(bin, leader, kWave);
          if (__ballot(on && bin == bin0) == act) {
            if ((int)(threadIdx.x & (kWave - 1)) == leader) atomicAdd(&lh[bin0], (uint32_t)__popcll(act));
          } else if (on) {
            atomicAdd(&lh[bin], 1u);
          }
        }
      } else {
        if (on) atomicAdd(&lh[bin], 1u);
      }
    }
    __syncthreads();
    cur = next_state<kSmallWG>(lh, bits, cur, scratch, &shared_state);
    __syncthreads();
  }
  const key_t T = (key_t)cur.prefix;
  const uint32_t take = cur.k_rem;
  uint32_t cnt = 0;  // low half: above, high half: equal
#pragma unroll
  for (int j = 0; j < kSmallKeys; ++j)
    if ((uint32_t)j < kpt && base + j < n) cnt += key[j] > T ? 1u : (key[j] == T ? (1u << 16) : 0u);
  uint32_t total;
  const uint32_t ex = workgroup_exclusive_scan<kSmallWG>(cnt, scratch, &total);
  uint32_t n_above = ex & 0xffffu, n_equal = ex >> 16;
#pragma unroll
  for (int j = 0; j < kSmallKeys; ++j) {
    if ((uint32_t)j >= kpt || base + j >= n) continue;
    if (key[j] > T) {
      const uint32_t pos = n_above + (n_equal < take ? n_equal : take);
      if (pos < k) out_idx[pos] = base + j;
      ++n_above;
    } else if (key[j] == T) {
      if (n_equal < take) {
        const uint32_t pos = n_above + n_equal;
        if (pos < k) out_idx[pos] = base + j;
      }
      ++n_equal;
    }
  }
}

// Polls a workgroup of the compaction spends on one window of predecessors before it counts
// the earlier tiles itself (each poll is a load from device memory plus a short sleep, about a
// microsecond).  A host-side setting so that a test can force the fallback.
static uint32_t g_spin_limit = 1u << 16;
static uint32_t g_compact_groups = kCompactMaxGroups;

static uint32_t clear_grid(uint32_t n_tiles) {
  const uint32_t words = (uint32_t)(sizeof(SelectWs) / 4) + n_tiles;
  const uint32_t g = (words + kWG * 8 - 1) / (kWG * 8);
  return g < 1 ? 1 : (g > 256 ? 256 : g);
}

// The ordered write, shared by selection and mask compaction.  k_select_clear must have run.
template <int SRC>
static void run_compaction(const KeyArgs src, uint32_t n, int passes, SelectWs* ws,
                           unsigned long long* tiles, uint32_t* out_idx, uint32_t out_cap,
                           uint32_t* out_count, hipStream_t st) {
  const uint32_t n_tiles = (uint32_t)n_tiles_of(n);
  uint32_t span = (n_tiles + g_compact_groups - 1) / g_compact_groups;  // 1 up to kCompactMaxGroups tiles
  if (span == 0) span = 1;
  launch((k_compact<SRC>), dim3((n_tiles + span - 1) / span), dim3(kWG), 0, st, src, n, n_tiles, span, passes, ws,
         tiles, out_idx, out_cap, out_count, g_spin_limit);
}

template <int SRC>
static void run_select(const KeyArgs scores, uint32_t n, uint32_t k, uint32_t* out_idx, void* workspace,
                       hipStream_t st) {
  if (n <= kSmallSelect) {
    if (n <= 8 * kSmallWG)
      launch((k_select_small<SRC, 8>), dim3(1), dim3(kSmallWG), 0, st, scores, n, k, out_idx);
    else
      launch((k_select_small<SRC, 16>), dim3(1), dim3(kSmallWG), 0, st, scores, n, k, out_idx);
    return;
  }
  SelectWs* ws = (SelectWs*)workspace;
  unsigned long long* tiles = (unsigned long long*)((char*)workspace + kWsTileOffset);
  const uint32_t n_tiles = (uint32_t)n_tiles_of(n);
  launch(k_select_clear, dim3(clear_grid(n_tiles)), dim3(kWG), 0, st, ws, (uint32_t)(sizeof(SelectWs) / 4), k,
         tiles, n_tiles);
  const uint32_t n_htiles = (uint32_t)(((uint64_t)n + kHistTileKeys - 1) / kHistTileKeys);
  // Every workgroup ends a pass with one global add per non-empty bin, so beyond a few
  // hundred workgroups more of them only add flush traffic: an eighth of the tiles, between
  // 256 and 2,048 (16.7 M float keys: 434 us with 16,384 workgroups, 192 us with 1,024; on the
  // benchmark's 2^20 keys a pass averages 9.4 us with 512 workgroups, 7.9 with 256, 9.0 with 128).
  uint32_t hgrid = n_htiles / 8;
  hgrid = hgrid < 256 ? 256 : (hgrid > 2048 ? 2048 : hgrid);
  if (hgrid > n_htiles) hgrid = n_htiles;
  const int passes = Key<SRC>::passes(scores);
  for (int p = 0; p < passes; ++p)
    launch((k_select_hist<SRC>), dim3(hgrid), dim3(kWG), 0, st, scores, n, n_htiles, p, ws);
  run_compaction<SRC>(scores, n, passes, ws, tiles, out_idx, k, nullptr, st);
}

__global__ void k_store_u32(uint32_t* __restrict__ p, uint32_t v) { *p = v; }

// Checking an index list (a debugging aid): one bit per block; an entry whose bit is already
// set is a repeat, an entry >= n_blocks is out of range.  counts[0] = out of range, counts[1] =
// repeats.
__global__ __launch_bounds__(kWG) void k_check_clear(uint32_t* __restrict__ bits, uint32_t n_words,
                                                     uint32_t* __restrict__ counts) {
  const uint32_t tid = blockIdx.x * kWG + threadIdx.x;
  for (uint32_t i = tid; i < n_words; i += gridDim.x * kWG) bits[i] = 0;
  if (tid < 2) counts[tid] = 0;
}
__global__ __launch_bounds__(kWG) void k_check_mark(const uint32_t* __restrict__ idx, uint32_t n_idx,
                                                    uint32_t n_blocks, uint32_t* __restrict__ bits,
                                                    uint32_t* __restrict__ counts) {
  uint32_t outside = 0, repeated = 0;
  for (uint64_t i = (uint64_t)blockIdx.x * kWG + threadIdx.x; i < n_idx; i += (uint64_t)gridDim.x * kWG) {
    const uint32_t b = idx[i];
    if (b >= n_blocks) {
      ++outside;
    } else {
      const uint32_t bit = 1u << (b & 31);
      if (atomicOr(&bits[b >> 5], bit) & bit) ++repeated;
    }
  }
  outside = wave_sum(outside), repeated = wave_sum(repeated);
  if ((threadIdx.x & (kWave - 1)) == 0) {
    if (outside) atomicAdd(&counts[0], outside);
    if (repeated) atomicAdd(&counts[1], repeated);
  }
}

// Round-robin strategy: the k blocks start, start+1, ... (mod n), written ascending.  When
// the run wraps, its wrapped head (blocks 0 .. wrap-1) comes first.
__global__ __launch_bounds__(kWG) void k_select_round(uint32_t n, uint32_t k, uint32_t start,
                                                      uint32_t* __restrict__ out_idx) {
  const uint32_t wrap = (uint64_t)start + k > n ? (uint32_t)((uint64_t)start + k - n) : 0;
  for (uint32_t i = blockIdx.x * kWG + threadIdx.x; i < k; i += gridDim.x * kWG)
    out_idx[i] = i < wrap ? i : start + (i - wrap);
}

}  // namespace scar

using namespace scar;

// Body of the scar_select_topk family once the arguments and the workspace are known.
// bounded: 64-bit integer scores are taken into [0, score_max].
static int select_topk_checked(int32_t score_type, const void* scores, uint32_t n_blocks, uint32_t k,
                               bool bounded, uint64_t score_max, uint32_t* out_idx, void* workspace,
                               hipStream_t st) {
  if (k == n_blocks) {  // a full checkpoint: every block, whatever the scores
    const uint32_t grid = (k + kWG - 1) / kWG < 4096 ? (k + kWG - 1) / kWG : 4096;
    launch(k_select_round, dim3(grid), dim3(kWG), 0, st, n_blocks, k, 0u, out_idx);
    return launch_status();
  }
  if (score_type == SCAR_SCORE_F32) {
    run_select<SRC_F32>(key_args(scores), n_blocks, k, out_idx, workspace, st);
    return launch_status();
  }
  KeyArgs a = key_args(scores);
  if (bounded) {  // keys in [0, score_max]: as many digits as score_max has
    int bits = 1;
    while (bits < 64 && (score_max >> bits) != 0) ++bits;
    a.passes = (bits + 10) / 11;
    a.bounded = 1;
    a.cap = score_max;
  }
  run_select<SRC_I64>(a, n_blocks, k, out_idx, workspace, st);
  return launch_status();
}

static int select_topk_args(int32_t score_type, const void* scores, uint32_t n_blocks, uint32_t k,
                            uint32_t* out_idx) {
  if (score_type != SCAR_SCORE_F32 && score_type != SCAR_SCORE_I64) return SCAR_ERR_INVALID_ARG;
  if (n_blocks > SCAR_MAX_BLOCKS || k > n_blocks) return SCAR_ERR_INVALID_ARG;
  if (k == 0) return SCAR_OK;
  if (!scores || !out_idx || !aligned(scores, score_type == SCAR_SCORE_I64 ? 8 : 4) ||
      !aligned(out_idx, 4))
    return SCAR_ERR_INVALID_ARG;
  return SCAR_OK;
}

extern "C" int scar_select_topk(int32_t score_type, const void* scores, uint32_t n_blocks, uint32_t k,
                                uint32_t* out_idx, void* workspace, size_t workspace_bytes,
                                void* stream) {
  int rc = select_topk_args(score_type, scores, n_blocks, k, out_idx);
  if (rc || k == 0) return rc;
  rc = check_workspace(workspace, workspace_bytes, n_blocks);
  if (rc) return rc;
  return select_topk_checked(score_type, scores, n_blocks, k, false, 0, out_idx, workspace,
                             (hipStream_t)stream);
}

extern "C" int scar_select_topk_bounded(int32_t score_type, const void* scores, uint32_t n_blocks,
                                        uint32_t k, uint64_t score_max, uint32_t* out_idx,
                                        void* workspace, size_t workspace_bytes, void* stream) {
  int rc = select_topk_args(score_type, scores, n_blocks, k, out_idx);
  if (rc || k == 0) return rc;
  rc = check_workspace(workspace, workspace_bytes, n_blocks);
  if (rc) return rc;
  return select_topk_checked(score_type, scores, n_blocks, k, true, score_max, out_idx, workspace,
                             (hipStream_t)stream);
}

extern "C" void scar_set_lookback_spin_limit(uint32_t polls) { g_spin_limit = polls; }

extern "C" void scar_set_compaction_groups(uint32_t groups) {
  g_compact_groups = (groups == 0 || groups > kCompactMaxGroups) ? kCompactMaxGroups : groups;
}

// ---- the selection for callers that cannot allocate -------------------------------------
// The scratch of scar_select_topk_static: one array per GPU, part of the loaded code object,
// sized for SCAR_STATIC_MAX_BLOCKS blocks.  In host code the array's name is only a handle;
// its device address is asked for once per device and kept.
static __device__ __align__(256) unsigned char scratch[workspace_bytes_for(SCAR_STATIC_MAX_BLOCKS)];

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device, or NULL.
static void* scratch_of_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}

extern "C" int scar_select_topk_static(int32_t score_type, const void* scores, uint32_t n_blocks,
                                       uint32_t k, uint32_t* out_idx, void* stream) {
  int rc = select_topk_args(score_type, scores, n_blocks, k, out_idx);
  if (rc) return rc;
  if (n_blocks > SCAR_STATIC_MAX_BLOCKS) return SCAR_ERR_WORKSPACE;
  if (k == 0) return SCAR_OK;
  void* ws = scratch_of_current_device();
  if (!ws) return SCAR_ERR_DEVICE;
  return select_topk_checked(score_type, scores, n_blocks, k, false, 0, out_idx, ws, (hipStream_t)stream);
}

extern "C" int scar_mask_to_indices(const uint8_t* mask, uint32_t n_blocks, uint32_t* out_idx,
                                    uint32_t* out_count, void* workspace, size_t workspace_bytes,
                                    void* stream) {
  if (n_blocks > SCAR_MAX_BLOCKS || !out_count || !aligned(out_count, 4)) return SCAR_ERR_INVALID_ARG;
  if (n_blocks && (!mask || !out_idx || !aligned(out_idx, 4))) return SCAR_ERR_INVALID_ARG;
  const int rc = check_workspace(workspace, workspace_bytes, n_blocks);
  if (rc) return rc;
  hipStream_t st = (hipStream_t)stream;
  SelectWs* ws = (SelectWs*)workspace;
  unsigned long long* tiles = (unsigned long long*)((char*)workspace + kWsTileOffset);
  const uint32_t n_tiles = (uint32_t)n_tiles_of(n_blocks);
  if (n_blocks == 0) {  // nothing to scan
    launch(k_store_u32, dim3(1), dim3(1), 0, st, out_count, 0u);
    return launch_status();
  }
  launch(k_select_clear, dim3(clear_grid(n_tiles)), dim3(kWG), 0, st, ws, (uint32_t)(sizeof(SelectWs) / 4), 0u,
         tiles, n_tiles);
  run_compaction<SRC_MASK>(key_args(mask), n_blocks, 0, ws, tiles, out_idx, n_blocks, out_count, st);
  return launch_status();
}

extern "C" int scar_select_round(uint32_t n_blocks, uint32_t k, uint64_t cursor, uint32_t* out_idx,
                                 void* stream) {
  if (n_blocks > SCAR_MAX_BLOCKS || k > n_blocks) return SCAR_ERR_INVALID_ARG;
  if (k == 0) return SCAR_OK;
  if (!out_idx || !aligned(out_idx, 4)) return SCAR_ERR_INVALID_ARG;
  const uint32_t grid = (k + kWG - 1) / kWG < 4096 ? (k + kWG - 1) / kWG : 4096;
  launch(k_select_round, dim3(grid), dim3(kWG), 0, (hipStream_t)stream, n_blocks, k,
                     (uint32_t)(cursor % n_blocks), out_idx);
  return launch_status();
}

extern "C" int scar_select_random(uint32_t n_blocks, uint32_t k, uint64_t seed, uint64_t draw,
                                  uint32_t* out_idx, void* workspace, size_t workspace_bytes,
                                  void* stream) {
  if (n_blocks > SCAR_MAX_BLOCKS || k > n_blocks) return SCAR_ERR_INVALID_ARG;
  if (k == 0) return SCAR_OK;
  if (!out_idx || !aligned(out_idx, 4)) return SCAR_ERR_INVALID_ARG;
  const int rc = check_workspace(workspace, workspace_bytes, n_blocks);
  if (rc) return rc;
  run_select<SRC_RANDOM>(key_args(nullptr, seed, draw), n_blocks, k, out_idx, workspace,
                         (hipStream_t)stream);
  return launch_status();
}

extern "C" size_t scar_check_workspace_bytes(uint64_t n_blocks) {
  return n_blocks > SCAR_MAX_BLOCKS ? 0 : ((n_blocks + 31) / 32 * 4 + 255) / 256 * 256 + 256;
}

extern "C" int scar_check_indices(const uint32_t* idx, uint32_t n_idx, uint32_t n_blocks, uint32_t* counts,
                                  void* workspace, size_t workspace_bytes, void* stream) {
  if (n_blocks > SCAR_MAX_BLOCKS || !counts || !aligned(counts, 4) || (n_idx && (!idx || !aligned(idx, 4))))
    return SCAR_ERR_INVALID_ARG;
  if (!workspace || !aligned(workspace, 256) || workspace_bytes < scar_check_workspace_bytes(n_blocks))
    return SCAR_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  const uint32_t n_words = (n_blocks + 31) / 32;
  const uint32_t cg = (n_words + kWG * 8 - 1) / (kWG * 8);
  launch(k_check_clear, dim3(cg < 1 ? 1 : (cg > 1024 ? 1024 : cg)), dim3(kWG), 0, st, (uint32_t*)workspace, n_words,
         counts);
  if (n_idx) {
    const uint32_t mg = (n_idx + kWG * 4 - 1) / (kWG * 4);
    launch(k_check_mark, dim3(mg > 4096 ? 4096 : mg), dim3(kWG), 0, st, idx, n_idx, n_blocks, (uint32_t*)workspace,
           counts);
  }
  return launch_status();
}
