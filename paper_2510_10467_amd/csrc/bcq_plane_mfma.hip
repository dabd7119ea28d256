#include "bcq_internal.hpp"

namespace bcq {
bool plane_mfma_supports(const GemmArgs &) { return false; }
hipError_t plane_mfma_launch(const GemmArgs &, hipStream_t) { return hipErrorNotSupported; }
}  // namespace bcq
