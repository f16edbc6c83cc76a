// Block-sparse attention backward for gfx950 (placeholder until the kernels land).
#include "asa_common.hpp"

namespace asa {

size_t bwd_workspace_bytes(const Problem &) { return 256; }

hipError_t launch_bwd(const Problem &, const void *, const void *, const void *, const void *,
                      const void *, const float *, const int32_t *, const int32_t *,
                      const int32_t *, const int32_t *, void *, void *, void *, void *,
                      hipStream_t) {
  return hipErrorNotSupported;
}

}  // namespace asa
