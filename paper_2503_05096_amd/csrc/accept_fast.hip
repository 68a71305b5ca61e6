// Register-resident acceptance kernel (placeholder until the kernel lands).
#include "adaspec_internal.h"

namespace adaspec {
bool accept_fast_path_supported(const adaspec_accept_dims &, const void *, const void *) { return false; }
hipError_t launch_accept_fast(const AcceptArgs &) { return hipErrorNotSupported; }
}  // namespace adaspec
