// Placeholder until the MFMA attention kernels land: reports "not supported" so callers use
// the generic kernels.
#include "internal.h"
namespace jpp {
bool attention_mfma_supported(const AttnDesc&) { return false; }
hipError_t launch_attention_fwd_mfma(const AttnDesc&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_attention_bwd_mfma(const AttnDesc&, hipStream_t) { return hipErrorNotSupported; }
}  // namespace jpp
