// Matrix-core Matching Pursuit encoder (placeholder until the kernel lands: reports unsupported).
#include "csr_internal.h"

namespace csr {

bool encode_mfma_supported(const EncodeArgs &) { return false; }
size_t encode_mfma_workspace_bytes(int32_t, int64_t, int32_t, int32_t) { return 0; }
hipError_t launch_encode_mfma(const EncodeArgs &) { return hipErrorNotSupported; }

}  // namespace csr
