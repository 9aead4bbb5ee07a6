// Chunked prefill of TreeKV for gfx950 (placeholder until the MFMA kernels land).
#include "treekv_internal.h"

namespace tkv {
int launch_prefill(const Params&, const void*, const void*, const void*, int, float*, int32_t*, int32_t*, int32_t*,
                   hipStream_t) {
  return TREEKV_EUNSUPPORTED;
}
}  // namespace tkv
