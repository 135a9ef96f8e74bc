// placeholder until the MFMA flash-attention kernels land
#include "kernels.h"
namespace tide {
bool attn_mfma_supported(const AttnArgs&) { return false; }
hipError_t launch_attn_fwd_mfma(const AttnArgs&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_attn_bwd_mfma(const AttnArgs&, hipStream_t) { return hipErrorNotSupported; }
}  // namespace tide
