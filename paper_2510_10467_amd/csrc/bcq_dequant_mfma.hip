// Large-batch kernel (placeholder until the fp16 MFMA path lands): reports
// that it supports nothing, so the dispatcher never selects it.
#include "bcq_internal.hpp"

namespace bcq {
bool dequant_mfma_supports(const GemmArgs &) { return false; }
hipError_t dequant_mfma_launch(const GemmArgs &, hipStream_t) { return hipErrorNotSupported; }
}  // namespace bcq
