// The persistent-storage leg (Section 4.3, checkpoint step 4 and recovery step 2): packed
// rows leave the GPU through a pinned host buffer and a writer thread puts them into the
// store file while the stream goes on with the next iteration.  Host code only.
#include <fcntl.h>
#include <sys/stat.h>
#include <unistd.h>

#include <condition_variable>
#include <cstring>
#include <deque>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

#include "../../include/scar_store.h"
#include "scar_host.hpp"

namespace {

constexpr uint64_t kDataOffset = 4096;
constexpr char kMagic[8] = {'S', 'C', 'A', 'R', 'S', 'T', 'O', '1'};

struct Header {
  char magic[8];
  int32_t dtype;
  uint32_t block_len;
  uint64_t n_elems;
  uint32_t row_bytes;
};

// Header of a store whose blocks differ in length; the (n_blocks + 1) element offsets follow
// at byte 4,096, the data after them on the next 4,096-byte boundary.
constexpr char kVarMagic[8] = {'S', 'C', 'A', 'R', 'S', 'T', 'V', '1'};
struct VarHeader {
  char magic[8];
  int32_t dtype;
  uint32_t n_blocks;
  uint64_t n_elems;
  uint64_t data_offset;
};

struct Slot {
  char* rows = nullptr;      // pinned, slot_bytes
  uint32_t* idx = nullptr;   // pinned, max_rows
  hipEvent_t copied = nullptr;
  uint32_t n = 0;
  uint64_t bytes = 0;        // of rows that were copied (stores with unequal blocks)
  bool busy = false;
};

int checkpoint_elem_bytes(int32_t dtype) { return (dtype == SCAR_BF16 || dtype == SCAR_F32_BF16C) ? 2 : 4; }

bool write_all(int fd, const char* p, size_t n, uint64_t off) {
  while (n) {
    const ssize_t w = pwrite(fd, p, n, (off_t)off);
    if (w <= 0) return false;
    p += w, n -= (size_t)w, off += (uint64_t)w;
  }
  return true;
}

bool read_all(int fd, char* p, size_t n, uint64_t off) {
  while (n) {
    const ssize_t r = pread(fd, p, n, (off_t)off);
    if (r <= 0) return false;
    p += r, n -= (size_t)r, off += (uint64_t)r;
  }
  return true;
}

}  // namespace

struct scar_store {
  int fd = -1;
  int device = 0;
  scar_layout layout{};
  uint64_t n_blocks = 0;
  uint32_t row_bytes = 0;
  uint32_t max_rows = 0;
  uint64_t slot_bytes = 0;            // capacity of a pinned row buffer
  uint64_t data_offset = kDataOffset; // of block 0 in the file
  std::vector<uint64_t> offsets;      // blocks of unequal length: n_blocks + 1 element offsets; else empty
  uint32_t elem_bytes = 4;
  Slot slot[2];
  std::mutex mu;
  std::condition_variable cv;
  std::deque<int> queue;  // slots handed to the writer, in order
  bool stop = false;
  bool failed = false;
  std::thread writer;

  // Bytes of block b that exist (the last block may be short).
  uint64_t block_bytes(uint64_t b) const {
    const uint64_t lo = b * layout.block_len;
    const uint64_t hi = lo + layout.block_len < layout.n_elems ? lo + layout.block_len : layout.n_elems;
    return (hi - lo) * (uint64_t)(row_bytes / layout.block_len);
  }

  bool is_var() const { return !offsets.empty(); }

  // Blocks of unequal length: the rows are packed in list order; runs of consecutive blocks
  // are consecutive in the file too and go out in one write.
  bool write_var_rows(const Slot& s) {
    uint64_t pos = 0;
    for (uint32_t i = 0; i < s.n;) {
      const uint32_t b = s.idx[i];
      if (b >= n_blocks) {
        ++i;
        continue;
      }
      uint32_t j = i + 1;
      while (j < s.n && s.idx[j] == s.idx[j - 1] + 1 && s.idx[j] < n_blocks) ++j;
      const uint64_t bytes = (offsets[s.idx[j - 1] + 1] - offsets[b]) * elem_bytes;
      if (pos + bytes > s.bytes) return false;  // the caller handed over fewer elements than the list needs
      if (bytes && !write_all(fd, s.rows + pos, bytes, data_offset + offsets[b] * elem_bytes)) return false;
      pos += bytes;
      i = j;
    }
    return true;
  }

  void write_slot(Slot& s) {
    bool ok = hipEventSynchronize(s.copied) == hipSuccess;
    if (is_var()) {
      ok = ok && write_var_rows(s);
      std::lock_guard<std::mutex> lock(mu);
      if (!ok) failed = true;
      s.busy = false;
      cv.notify_all();
      return;
    }
    for (uint32_t i = 0; ok && i < s.n;) {
      // consecutive full blocks go out in one write
      const uint32_t b = s.idx[i];
      if (b >= n_blocks) {
        ++i;
        continue;
      }
      uint32_t j = i + 1;
      while (j < s.n && s.idx[j] == s.idx[j - 1] + 1 && s.idx[j] < n_blocks &&
             block_bytes(s.idx[j - 1]) == row_bytes)
        ++j;
      const uint64_t bytes = (uint64_t)(j - i - 1) * row_bytes + block_bytes(s.idx[j - 1]);
      ok = write_all(fd, s.rows + (uint64_t)i * row_bytes, bytes, kDataOffset + (uint64_t)b * row_bytes);
      i = j;
    }
    std::lock_guard<std::mutex> lock(mu);
    if (!ok) failed = true;
    s.busy = false;
    cv.notify_all();
  }

  void run() {
    (void)hipSetDevice(device);
    for (;;) {
      int k;
      {
        std::unique_lock<std::mutex> lock(mu);
        cv.wait(lock, [&] { return stop || !queue.empty(); });
        if (queue.empty()) return;  // stop requested and nothing left
        k = queue.front();
        queue.pop_front();
      }
      write_slot(slot[k]);
    }
  }
};

namespace {

// max_elems: capacity of a pinned row buffer in elements for stores with unequal blocks
// (fixed-length stores: max_rows rows).
int finish_open(scar_store* s, uint32_t max_rows, scar_store** out, uint64_t max_elems = 0) {
  s->elem_bytes = (uint32_t)checkpoint_elem_bytes(s->layout.dtype);
  if (!s->is_var()) s->row_bytes = s->layout.block_len * s->elem_bytes;
  s->max_rows = max_rows;
  s->slot_bytes = s->is_var() ? max_elems * s->elem_bytes : (uint64_t)max_rows * s->row_bytes;
  bool ok = hipGetDevice(&s->device) == hipSuccess;
  for (Slot& sl : s->slot) {
    ok = ok && hipHostMalloc((void**)&sl.rows, (size_t)s->slot_bytes + 16, hipHostMallocDefault) == hipSuccess;
    ok = ok && hipHostMalloc((void**)&sl.idx, (size_t)max_rows * 4 + 16, hipHostMallocDefault) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&sl.copied, hipEventDisableTiming) == hipSuccess;
  }
  if (!ok) {
    for (Slot& sl : s->slot) {
      if (sl.rows) (void)hipHostFree(sl.rows);
      if (sl.idx) (void)hipHostFree(sl.idx);
      if (sl.copied) (void)hipEventDestroy(sl.copied);
    }
    close(s->fd);
    delete s;
    return SCAR_ERR_DEVICE;
  }
  try {
    s->writer = std::thread([s] { s->run(); });
  } catch (...) {  // no thread to be had: undo everything, nothing leaves this call but a status
    for (Slot& sl : s->slot) {
      (void)hipHostFree(sl.rows);
      (void)hipHostFree(sl.idx);
      (void)hipEventDestroy(sl.copied);
    }
    close(s->fd);
    delete s;
    return SCAR_ERR_DEVICE;
  }
  *out = s;
  return SCAR_OK;
}

}  // namespace

extern "C" int scar_store_create(const char* path, const scar_layout* layout, uint32_t max_rows,
                                 scar_store** out) {
  const uint64_t nb = scar::layout_blocks(layout);
  if (!path || !out || nb == UINT64_MAX || max_rows == 0) return SCAR_ERR_INVALID_ARG;
  if ((uint64_t)layout->block_len * checkpoint_elem_bytes(layout->dtype) > 0xffffffffull)
    return SCAR_ERR_INVALID_ARG;
  scar_store* s = new (std::nothrow) scar_store;
  if (!s) return SCAR_ERR_DEVICE;
  s->layout = *layout;
  s->n_blocks = nb;
  s->fd = open(path, O_RDWR | O_CREAT | O_TRUNC, 0644);
  Header h{};
  std::memcpy(h.magic, kMagic, 8);
  h.dtype = layout->dtype;
  h.block_len = layout->block_len;
  h.n_elems = layout->n_elems;
  h.row_bytes = layout->block_len * (uint32_t)checkpoint_elem_bytes(layout->dtype);
  const uint64_t size = kDataOffset + layout->n_elems * (uint64_t)checkpoint_elem_bytes(layout->dtype);
  if (s->fd < 0 || !write_all(s->fd, (const char*)&h, sizeof h, 0) || ftruncate(s->fd, (off_t)size) != 0) {
    if (s->fd >= 0) close(s->fd);
    delete s;
    return SCAR_ERR_IO;
  }
  return finish_open(s, max_rows, out);
}

extern "C" int scar_store_open(const char* path, uint32_t max_rows, scar_layout* layout_out,
                               scar_store** out) {
  if (!path || !out || max_rows == 0) return SCAR_ERR_INVALID_ARG;
  scar_store* s = new (std::nothrow) scar_store;
  if (!s) return SCAR_ERR_DEVICE;
  s->fd = open(path, O_RDWR);
  Header h{};
  if (s->fd < 0 || !read_all(s->fd, (char*)&h, sizeof h, 0) || std::memcmp(h.magic, kMagic, 8) != 0) {
    if (s->fd >= 0) close(s->fd);
    delete s;
    return SCAR_ERR_IO;
  }
  s->layout.dtype = h.dtype;
  s->layout.block_len = h.block_len;
  s->layout.n_elems = h.n_elems;
  s->n_blocks = scar::layout_blocks(&s->layout);
  if (s->n_blocks == UINT64_MAX ||
      h.row_bytes != h.block_len * (uint32_t)checkpoint_elem_bytes(h.dtype)) {
    close(s->fd);
    delete s;
    return SCAR_ERR_IO;
  }
  if (layout_out) *layout_out = s->layout;
  return finish_open(s, max_rows, out);
}

extern "C" int scar_store_save_async(scar_store* s, const void* staging, const uint32_t* idx,
                                     uint32_t n_idx, void* stream) {
  if (!s || s->is_var() || n_idx > s->max_rows) return SCAR_ERR_INVALID_ARG;
  if (n_idx == 0) return SCAR_OK;
  if (!staging || !idx) return SCAR_ERR_INVALID_ARG;
  int k;
  {
    std::unique_lock<std::mutex> lock(s->mu);
    s->cv.wait(lock, [&] { return !s->slot[0].busy || !s->slot[1].busy; });
    k = s->slot[0].busy ? 1 : 0;
    s->slot[k].busy = true;
  }
  Slot& sl = s->slot[k];
  sl.n = n_idx;
  hipStream_t st = (hipStream_t)stream;
  bool ok = hipMemcpyAsync(sl.idx, idx, (size_t)n_idx * 4, hipMemcpyDeviceToHost, st) == hipSuccess;
  ok = ok && hipMemcpyAsync(sl.rows, staging, (size_t)n_idx * s->row_bytes, hipMemcpyDeviceToHost, st) == hipSuccess;
  ok = ok && hipEventRecord(sl.copied, st) == hipSuccess;
  // A copy that was enqueued before a later step failed may still be writing into the pinned
  // buffer: the slot is handed back only once the stream has passed it.
  if (!ok) (void)hipStreamSynchronize(st);
  std::lock_guard<std::mutex> lock(s->mu);
  if (!ok) {
    sl.busy = false;
    s->cv.notify_all();
    return SCAR_ERR_DEVICE;
  }
  s->queue.push_back(k);
  s->cv.notify_all();
  return SCAR_OK;
}

extern "C" int scar_store_wait(scar_store* s) {
  if (!s) return SCAR_ERR_INVALID_ARG;
  bool failed;
  {
    std::unique_lock<std::mutex> lock(s->mu);
    s->cv.wait(lock, [&] { return s->queue.empty() && !s->slot[0].busy && !s->slot[1].busy; });
    failed = s->failed;
    s->failed = false;
  }
  if (fsync(s->fd) != 0) failed = true;
  return failed ? SCAR_ERR_IO : SCAR_OK;
}

extern "C" int scar_store_load(scar_store* s, const uint32_t* idx_host, uint32_t n_idx, void* rows,
                               void* stream) {
  if (!s || s->is_var() || n_idx > s->max_rows) return SCAR_ERR_INVALID_ARG;
  if (n_idx == 0) return SCAR_OK;
  if (!idx_host || !rows) return SCAR_ERR_INVALID_ARG;
  const int rc = scar_store_wait(s);  // both pinned buffers are free afterwards
  if (rc) return rc;
  Slot& sl = s->slot[0];
  for (uint32_t i = 0; i < n_idx; ++i) {
    const uint32_t b = idx_host[i];
    if (b >= s->n_blocks) return SCAR_ERR_INVALID_ARG;
    char* dst = sl.rows + (uint64_t)i * s->row_bytes;
    const uint64_t bytes = s->block_bytes(b);
    if (!read_all(s->fd, dst, bytes, kDataOffset + (uint64_t)b * s->row_bytes)) return SCAR_ERR_IO;
    if (bytes < s->row_bytes) std::memset(dst + bytes, 0, s->row_bytes - bytes);
  }
  hipStream_t st = (hipStream_t)stream;
  if (hipMemcpyAsync(rows, sl.rows, (size_t)n_idx * s->row_bytes, hipMemcpyHostToDevice, st) != hipSuccess ||
      hipStreamSynchronize(st) != hipSuccess)
    return SCAR_ERR_DEVICE;
  return SCAR_OK;
}

// ---- stores whose blocks differ in length (by-layer partitioning, Section 5.1) -------------

extern "C" int scar_var_store_create(const char* path, int32_t dtype, uint32_t n_blocks,
                                     const uint64_t* offsets_host, uint32_t max_rows, uint64_t max_elems,
                                     scar_store** out) {
  if (!path || !out || !offsets_host || n_blocks == 0 || n_blocks > SCAR_MAX_BLOCKS || max_rows == 0 ||
      max_elems == 0 || !scar::dtype_ok(dtype) || offsets_host[0] != 0)
    return SCAR_ERR_INVALID_ARG;
  for (uint32_t b = 0; b < n_blocks; ++b)
    if (offsets_host[b + 1] < offsets_host[b]) return SCAR_ERR_INVALID_ARG;
  scar_store* s = new (std::nothrow) scar_store;
  if (!s) return SCAR_ERR_DEVICE;
  s->layout.dtype = dtype;
  s->layout.block_len = 1;
  s->layout.n_elems = offsets_host[n_blocks];
  s->n_blocks = n_blocks;
  s->offsets.assign(offsets_host, offsets_host + n_blocks + 1);
  const uint64_t table = ((uint64_t)(n_blocks + 1) * 8 + kDataOffset - 1) / kDataOffset * kDataOffset;
  s->data_offset = kDataOffset + table;
  VarHeader h{};
  std::memcpy(h.magic, kVarMagic, 8);
  h.dtype = dtype;
  h.n_blocks = n_blocks;
  h.n_elems = s->layout.n_elems;
  h.data_offset = s->data_offset;
  const uint64_t size = s->data_offset + s->layout.n_elems * (uint64_t)checkpoint_elem_bytes(dtype);
  s->fd = open(path, O_RDWR | O_CREAT | O_TRUNC, 0644);
  if (s->fd < 0 || !write_all(s->fd, (const char*)&h, sizeof h, 0) ||
      !write_all(s->fd, (const char*)s->offsets.data(), (size_t)(n_blocks + 1) * 8, kDataOffset) ||
      ftruncate(s->fd, (off_t)size) != 0) {
    if (s->fd >= 0) close(s->fd);
    delete s;
    return SCAR_ERR_IO;
  }
  return finish_open(s, max_rows, out, max_elems);
}

extern "C" int scar_var_store_save_async(scar_store* s, const void* staging, uint64_t staging_elems,
                                         const uint32_t* idx, uint32_t n_idx, void* stream) {
  if (!s || !s->is_var() || n_idx > s->max_rows || staging_elems * s->elem_bytes > s->slot_bytes)
    return SCAR_ERR_INVALID_ARG;
  if (n_idx == 0) return SCAR_OK;
  if (!idx || (staging_elems && !staging)) return SCAR_ERR_INVALID_ARG;
  int k;
  {
    std::unique_lock<std::mutex> lock(s->mu);
    s->cv.wait(lock, [&] { return !s->slot[0].busy || !s->slot[1].busy; });
    k = s->slot[0].busy ? 1 : 0;
    s->slot[k].busy = true;
  }
  Slot& sl = s->slot[k];
  sl.n = n_idx;
  sl.bytes = staging_elems * s->elem_bytes;
  hipStream_t st = (hipStream_t)stream;
  bool ok = hipMemcpyAsync(sl.idx, idx, (size_t)n_idx * 4, hipMemcpyDeviceToHost, st) == hipSuccess;
  if (sl.bytes) ok = ok && hipMemcpyAsync(sl.rows, staging, (size_t)sl.bytes, hipMemcpyDeviceToHost, st) == hipSuccess;
  ok = ok && hipEventRecord(sl.copied, st) == hipSuccess;
  if (!ok) (void)hipStreamSynchronize(st);  // a copy already enqueued may still be writing into the slot
  std::lock_guard<std::mutex> lock(s->mu);
  if (!ok) {
    sl.busy = false;
    s->cv.notify_all();
    return SCAR_ERR_DEVICE;
  }
  s->queue.push_back(k);
  s->cv.notify_all();
  return SCAR_OK;
}

extern "C" int scar_var_store_load(scar_store* s, const uint32_t* idx_host, uint32_t n_idx, void* rows,
                                   uint64_t* row_offsets, void* stream) {
  if (!s || !s->is_var() || n_idx > s->max_rows || !row_offsets) return SCAR_ERR_INVALID_ARG;
  if (n_idx && (!idx_host || !rows)) return SCAR_ERR_INVALID_ARG;
  const int rc = scar_store_wait(s);  // both pinned buffers are free afterwards
  if (rc) return rc;
  Slot& sl = s->slot[0];
  // the offsets travel through the second slot's row buffer (8 bytes per listed block + 8)
  uint64_t* offs = (uint64_t*)s->slot[1].rows;
  if ((uint64_t)(n_idx + 1) * 8 > s->slot_bytes + 16) return SCAR_ERR_INVALID_ARG;
  uint64_t pos = 0;
  for (uint32_t i = 0; i < n_idx; ++i) {
    const uint32_t b = idx_host[i];
    if (b >= s->n_blocks) return SCAR_ERR_INVALID_ARG;
    const uint64_t bytes = (s->offsets[b + 1] - s->offsets[b]) * s->elem_bytes;
    if (pos + bytes > s->slot_bytes) return SCAR_ERR_INVALID_ARG;
    if (bytes && !read_all(s->fd, sl.rows + pos, bytes, s->data_offset + s->offsets[b] * s->elem_bytes))
      return SCAR_ERR_IO;
    offs[i] = pos / s->elem_bytes;
    pos += bytes;
  }
  offs[n_idx] = pos / s->elem_bytes;
  hipStream_t st = (hipStream_t)stream;
  bool ok = hipMemcpyAsync(row_offsets, offs, (size_t)(n_idx + 1) * 8, hipMemcpyHostToDevice, st) == hipSuccess;
  if (pos) ok = ok && hipMemcpyAsync(rows, sl.rows, (size_t)pos, hipMemcpyHostToDevice, st) == hipSuccess;
  ok = (hipStreamSynchronize(st) == hipSuccess) && ok;
  return ok ? SCAR_OK : SCAR_ERR_DEVICE;
}

extern "C" int scar_store_close(scar_store* s) {
  if (!s) return SCAR_ERR_INVALID_ARG;
  const int rc = scar_store_wait(s);
  {
    std::lock_guard<std::mutex> lock(s->mu);
    s->stop = true;
    s->cv.notify_all();
  }
  s->writer.join();
  for (Slot& sl : s->slot) {
    (void)hipHostFree(sl.rows);
    (void)hipHostFree(sl.idx);
    (void)hipEventDestroy(sl.copied);
  }
  close(s->fd);
  delete s;
  return rc;
}
