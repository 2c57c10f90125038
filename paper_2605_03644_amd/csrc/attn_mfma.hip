// bf16 MFMA query-over-cache attention (placeholder until the tiled kernel lands).
#include "adapshot_internal.h"

namespace adapshot {
bool attn_mfma_supported(const adapshot_model_desc&) { return false; }
hipError_t launch_attn_mfma(const AttnParams&, hipStream_t) { return hipErrorNotSupported; }
}  // namespace adapshot
