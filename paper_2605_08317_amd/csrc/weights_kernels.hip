// Stage 1 of Alg. 1 (placeholder until the MFMA kernels land).
#include "rdkv_internal.h"

namespace rdkv {

size_t weights_scratch_floats(const rdkv_config&, int64_t) { return 16; }

hipError_t launch_weights(const rdkv_config&, const int64_t*, const int32_t*, const std::vector<int32_t>&,
                          const uint16_t*, const uint16_t*, float*, float*, float*, hipStream_t) {
  return hipErrorNotSupported;
}

}  // namespace rdkv
