// bf16 MFMA LM head (placeholder until the kernel lands).
#include "common.hpp"
#include "launch.hpp"
namespace aurora {
bool lmhead_mfma_supported(const AcceptLaunch&) { return false; }
int lmhead_mfma_stat_tile() { return 256; }
hipError_t launch_lmhead_mfma(const AcceptLaunch&, hipStream_t) { return hipErrorNotSupported; }
}  // namespace aurora
