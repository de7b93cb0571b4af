// placeholder, replaced below
#include "moe_internal.h"
extern "C" {
int64_t moe_static_workspace_bytes(const moe_handle_t *h, int32_t T, int32_t capacity, int32_t mode) { moe355::set_error("not built yet"); return MOE_ERR_UNSUPPORTED; }
int moe_layer_forward_static(moe_handle_t *h, const void *x, const void *wg, const float *gate_bias,
                             const void *w1, const void *w2, const void *b1, const void *b2,
                             int32_t T, int32_t capacity, int32_t mode, void *y,
                             int32_t *dropped_count, const moe_routing_t *routing_out,
                             void *workspace, int64_t workspace_bytes, void *stream) { moe355::set_error("not built yet"); return MOE_ERR_UNSUPPORTED; }
}
