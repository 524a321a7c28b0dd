// bf16 MFMA mixed attention (placeholder: reports unsupported so that the dispatcher uses
// the type-generic kernel).
#include "flexco_internal.h"

namespace flexco {
int32_t launch_attention_mfma(const flexco_layer_cfg&, const flexco_maps&, const void*, size_t,
                              const flexco_kv_pool&, float*, float*, hipStream_t) {
  return FLEXCO_EUNSUPPORTED;
}
}  // namespace flexco
