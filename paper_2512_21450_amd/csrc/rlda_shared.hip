// Shared-prefix MFMA path (placeholder until the kernels land).
#include "rlda_internal.h"

namespace rlda {
bool shared_supported(const rlda_desc&) { return false; }
size_t shared_workspace_bytes(const rlda_desc&) { return 0; }
hipError_t launch_shared(const rlda_desc&, hipStream_t) { return hipErrorNotSupported; }
}  // namespace rlda
