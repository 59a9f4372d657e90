// Stage (c), MFMA path placeholder: filled in by the bf16 kernel.
#include "dr_internal.h"
namespace dr {
bool attn_mfma_supported(const AttnArgs&) { return false; }
hipError_t launch_attn_mfma(const AttnArgs&, hipStream_t) { return hipErrorNotSupported; }
}  // namespace dr
