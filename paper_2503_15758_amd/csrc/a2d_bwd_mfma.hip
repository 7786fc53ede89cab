// bf16 MFMA backward tile kernels (placeholder: not yet covering any shape, so the
// C-ABI layer routes every backward call to the generic kernels).
#include "a2d_common.hpp"

namespace a2d {

bool bwd_mfma_supported(const a2d_tile_desc&) { return false; }

hipError_t launch_bwd_mfma(const a2d_tile_desc&, const void*, const void*, const void*, const void*,
                           const float*, const float*, float*, float*, float*, hipStream_t) {
  return hipErrorNotSupported;
}

}  // namespace a2d
