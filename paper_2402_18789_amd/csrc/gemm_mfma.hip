// bf16 MFMA projections (placeholder until the tiled kernel lands: reports unsupported so
// that the dispatcher uses the type-generic kernel).
#include "flexco_internal.h"

namespace flexco {
int32_t launch_gemm_mfma(const void*, const void*, void*, const void*, const void*, int, int, int, size_t, size_t,
                         size_t, size_t, bool, hipStream_t) {
  return FLEXCO_EUNSUPPORTED;
}
}  // namespace flexco
