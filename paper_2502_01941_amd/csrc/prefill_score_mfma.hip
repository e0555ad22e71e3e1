// Window-attention softmax partials on the matrix cores (placeholder until the kernel lands).
#include "common.hpp"

namespace shotkv {

bool score_uses_mfma(const PrefillDims&) { return false; }

hipError_t launch_score_partials_mfma(const PrefillDims&, const void*, const void*,
                                      const PrefillWorkspace&, hipStream_t) {
  return hipErrorNotSupported;
}

}  // namespace shotkv
