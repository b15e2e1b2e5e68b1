// MFMA path (bf16 matrix-core kernels).  Placeholder until the kernels land: reports that no
// configuration is covered, so every handle is served by the generic path.
#include "hla_handle.h"

namespace hla {

bool mfma_supported(const hla_config&) { return false; }
hla_status mfma_workspace_plan(hla_handle*) { return HLA_ERR_UNSUPPORTED; }
hla_status mfma_set_weights(hla_handle*, hipStream_t) { return HLA_ERR_UNSUPPORTED; }
hla_status mfma_forward(hla_handle*, const hla_call_args&) { return HLA_ERR_UNSUPPORTED; }
hla_status mfma_backward(hla_handle*, const hla_call_args&) { return HLA_ERR_UNSUPPORTED; }

}  // namespace hla
