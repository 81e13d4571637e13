// placeholder until the UKAN path lands
#include "kan.h"
extern "C" size_t ukan_workspace_bytes(const ukan_layer_desc *, int64_t, int32_t, int) { return 0; }
extern "C" int ukan_cg_forward(const ukan_layer_desc *, int64_t, const float *, const ukan_params *, float *, int32_t, void *, size_t, void *) { return KAN_ERR_UNSUPPORTED; }
extern "C" int ukan_cg_backward(const ukan_layer_desc *, int64_t, const float *, const ukan_params *, const float *, float *, const ukan_grads *, int32_t, void *, size_t, void *) { return KAN_ERR_UNSUPPORTED; }
extern "C" int ukan_group_index(const ukan_layer_desc *, int64_t, const float *, int32_t *, int32_t *, int32_t *, void *) { return KAN_ERR_UNSUPPORTED; }
