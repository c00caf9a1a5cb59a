// bf16 matrix-core backward kernel for GDPA (placeholder until the fused kernel lands: the
// generic kernels serve the backward pass).
#include "common.h"

namespace kunlun {

bool mfma_bwd_supported(const AttnParams&, int) { return false; }
size_t mfma_bwd_workspace_tail(int, int, int, int, int64_t) { return 0; }
hipError_t launch_mfma_bwd(const AttnParams&, void*, hipStream_t) { return hipErrorNotSupported; }

}  // namespace kunlun
