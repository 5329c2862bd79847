// Grouped-query chunk kernel (MFMA path) -- placeholder until the kernel lands.
#include "fd_internal.h"

namespace fd {
hipError_t launch_partial_unified_gqa(const Problem &, hipStream_t) { return hipErrorNotSupported; }
}  // namespace fd
