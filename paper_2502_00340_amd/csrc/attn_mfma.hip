// placeholder until the MFMA attention backward lands
#include "common.h"
namespace cf {
bool attn_mfma_supported(const cf_layer_desc&) { return false; }
hipError_t launch_attn_bwd_mfma(const cf_layer_desc&, float, const void*, const void*, const void*,
                                const float*, const void*, const float*, const int32_t*,
                                const int32_t*, int, void*, void*, void*, hipStream_t) {
    return hipErrorNotSupported;
}
}  // namespace cf
