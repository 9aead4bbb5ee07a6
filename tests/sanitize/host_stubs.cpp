// Stand-ins for the kernel launchers, so that the host side of the C ABI (configuration checks, workspace
// carving, argument checks) can be linked and run under AddressSanitizer / UBSan without the kernels.
// Test infrastructure; never part of libtreekv.so.
#include "treekv_internal.h"

namespace tkv {
bool decode_shape_fits(const Params& p) { return p.cap <= 8192; }
int launch_decode(const Params&, const void*, const void*, const void*, float*, int32_t*, int32_t*, int32_t*, hipStream_t) { return TREEKV_OK; }
int launch_prefill(const Params&, const void*, const void*, const void*, int, float*, int32_t*, int32_t*, int32_t*, hipStream_t) { return TREEKV_OK; }
int launch_prompt(const Params&, const void*, const void*, const void*, int, int, int32_t*, int32_t*, int32_t*, float*, hipStream_t) { return TREEKV_OK; }
size_t prompt_blocks_lds(int, int, int, int, int) { return 0; }
int launch_wavelet(const float*, const void*, int, int, int, int, int, float*, float*, hipStream_t) { return TREEKV_OK; }
}  // namespace tkv
