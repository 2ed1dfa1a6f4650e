// bf16 attention on the matrix cores (placeholder until the tiled kernels land: nothing is
// routed here yet, attention runs on the vector-ALU kernels).
#include "kernels.hpp"

namespace k2bw {

bool attention_mfma_supported(const AttnDesc&) { return false; }

hipError_t attention_fwd_mfma(const AttnDesc&, const void*, void*, float*, hipStream_t) {
  return hipErrorInvalidValue;
}
hipError_t attention_bwd_mfma(const AttnDesc&, const void*, const void*, const float*, const void*, void*, float*,
                              hipStream_t) {
  return hipErrorInvalidValue;
}

}  // namespace k2bw
