#include "pd_internal.h"
namespace pd {
bool attn_prefill_mfma_supported(const AttnArgs &) { return false; }
hipError_t launch_attn_prefill_mfma(const AttnArgs &, hipStream_t) { return hipErrorNotSupported; }
}  // namespace pd
