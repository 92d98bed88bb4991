// Host-only entry points: sizes and messages.
#include "scar_host.hpp"

using namespace scar;

extern "C" uint64_t scar_n_blocks(const scar_layout* layout) {
  const uint64_t nb = layout_blocks(layout);
  return nb == UINT64_MAX ? 0 : nb;
}

extern "C" size_t scar_workspace_bytes(uint64_t n_blocks) {
  return n_blocks > SCAR_MAX_BLOCKS ? 0 : workspace_bytes_for(n_blocks);
}

extern "C" const char* scar_strerror(int status) {
  switch (status) {
    case SCAR_OK: return "ok";
    case SCAR_ERR_INVALID_ARG: return "invalid argument";
    case SCAR_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case SCAR_ERR_DEVICE: return "HIP reported an error while enqueueing";
    case -4: return "store file could not be created, opened, read or written";
    case SCAR_ERR_UNSUPPORTED: return "valid arguments, but this store type is not built for this call";
    default: return "unknown status";
  }
}
