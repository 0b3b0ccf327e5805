// bf16 MFMA chunk attention (placeholder until the kernel lands): reports "not supported" so the
// dispatcher takes the generic path.
#include "common.hpp"
#include "launch.hpp"
namespace aurora {
bool attn_mfma_supported(const AttnLaunch&) { return false; }
hipError_t launch_attn_mfma(const AttnLaunch&, hipStream_t) { return hipErrorNotSupported; }
}  // namespace aurora
