// Layer-stack driver (placeholder until the MFMA GEMMs land).
#include "stack.h"
extern "C" {
size_t climber_workspace_bytes(const climber_config *, int64_t) { return 0; }
int climber_layer_forward(const climber_config *, const climber_layer_weights *, const float *, int32_t, int32_t, climber_kv_cache *, const float *, float *, const int32_t *, const int32_t *, const int32_t *, int32_t, int32_t, void *, size_t, void *) { return CLIMBER_ERR_UNSUPPORTED; }
int climber_history_encode(const climber_config *, const climber_weights *, const float *, const void *, const int32_t *, const int32_t *, climber_kv_cache *, void *, size_t, void *) { return CLIMBER_ERR_UNSUPPORTED; }
int climber_sumi_score(const climber_config *, const climber_weights *, const float *, const climber_kv_cache *, const void *, const int32_t *, int32_t, int32_t, const int32_t *, const int32_t *, float *, void *, size_t, void *) { return CLIMBER_ERR_UNSUPPORTED; }
}
