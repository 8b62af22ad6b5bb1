// Whole-network forward passes (placeholder until the assemblies land).
#include "common.h"

extern "C" size_t ds_forward_workspace(const ds_net* net, int32_t B) { (void)net; (void)B; return 0; }

extern "C" int32_t ds_forward(const ds_net* net, const void* images, int32_t B, const int32_t* route_override,
                              const float* logit_bias, float* logits, int32_t* routes_out, void* ws, size_t ws_bytes,
                              void* stream) {
    DS_FAIL(DS_EUNSUPPORTED, "ds_forward: not built yet");
}
