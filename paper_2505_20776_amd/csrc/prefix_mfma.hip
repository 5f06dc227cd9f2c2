// Prefix pass of Hybrid Tree Attention on the matrix cores (placeholder until the MFMA kernel lands).
#include "common.h"

namespace specext {

bool prefix_mfma_supports(const AttnParams&) { return false; }
hipError_t launch_prefix_mfma(const AttnParams&, hipStream_t) { return hipErrorNotSupported; }

}  // namespace specext
