// Placeholder until the chunked MFMA kernel lands: reports no supported shape so that every prefill takes the
// shape-agnostic kernel.
#include "quamba_internal.h"

namespace quamba {
bool prefill_mfma_supports(const quamba_ssd_shape_t &) { return false; }
hipError_t launch_prefill_mfma(const SsdArgs &, hipStream_t) { return hipErrorNotSupported; }
}  // namespace quamba
