// placeholder
#include "ctx.h"
extern "C" {
ssdt_status ssdt_layer_workspace(const ssdt_layer_desc *, size_t *, size_t *) { return SSDT_E_UNSUPPORTED; }
ssdt_status ssdt_layer_fwd(ssdt_ctx *, const ssdt_layer_desc *, const ssdt_layer_weights *, int32_t, const void *,
                           const void *, const int32_t *, void **, ssdt_layer_saved *, void *, size_t, ssdt_stream) { return SSDT_E_UNSUPPORTED; }
ssdt_status ssdt_layer_bwd(ssdt_ctx *, const ssdt_layer_desc *, const ssdt_layer_weights *, const ssdt_layer_saved *,
                           const int32_t *, const void *, void *, void *, const ssdt_layer_weights *, void *, size_t,
                           ssdt_stream) { return SSDT_E_UNSUPPORTED; }
}
