// bf16 flash-style attention for gfx950 (placeholder until the MFMA kernels land: reports
// "unsupported" so the generic kernels are used).
#include <hip/hip_runtime.h>

#include "device_math.h"
#include "kernels.h"

namespace tpl {
bool attn_bf16_supported(const AttnArgs&) { return false; }
hipError_t attn_bf16_fwd(const AttnArgs&) { return hipErrorNotSupported; }
hipError_t attn_bf16_bwd(const AttnArgs&) { return hipErrorNotSupported; }
}  // namespace tpl
