// Fused single-pass path (placeholder until the MFMA kernel lands).
#include "nadmm_internal.h"

namespace nadmm {

bool fused_supported(const Shape&, int64_t) { return false; }
int fused_num_partials(const Shape&) { return 0; }
size_t fused_pack_bytes(const Shape&) { return 0; }
hipError_t launch_fused(const RowArgs&, float*, void*, hipStream_t) { return hipErrorNotSupported; }

}  // namespace nadmm
