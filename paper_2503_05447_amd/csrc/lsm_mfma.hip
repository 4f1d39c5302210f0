// MFMA kernel family (bf16 operands, fp32 accumulation).  Placeholder until the kernels land:
// every shape is routed to the generic family.
#include "lsm_internal.h"
namespace lsm {
bool mfma_supported(const Dims&) { return false; }
size_t mfma_fwd_workspace(const Dims&) { return 0; }
size_t mfma_bwd_workspace(const Dims&) { return 0; }
hipError_t mfma_fwd(const Dims&, const FwdArgs&) { return hipErrorNotSupported; }
hipError_t mfma_bwd(const Dims&, const BwdArgs&) { return hipErrorNotSupported; }
}  // namespace lsm
