// Matrix-core verification attention (placeholder until the kernel lands).
#include "adaspec_internal.h"

namespace adaspec {
bool attn_fast_path_supported(const adaspec_attn_dims &) { return false; }
hipError_t launch_attn_mfma(const AttnArgs &) { return hipErrorNotSupported; }
}  // namespace adaspec
