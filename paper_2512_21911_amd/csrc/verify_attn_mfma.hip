// Verification attention, matrix-core kernel for bf16 inputs with head dimension 128.
#include "svf_device.h"

namespace svf {

bool mfma_supported(const svf_shape_t&) { return false; }
int mfma_splits(const svf_shape_t&) { return 1; }
hipError_t launch_verify_attn_mfma(const AttnParams&, hipStream_t) { return hipErrorNotSupported; }

}  // namespace svf
