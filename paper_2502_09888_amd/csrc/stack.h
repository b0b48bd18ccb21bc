// Internal interface between the C-ABI translation unit and the layer-stack driver.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/climber.h"

namespace climber {

// Attention with explicit row strides (q, k, v share one stride: they are column blocks of one
// fused projection output in the stack, dense arrays in the attention-only calls).
int attn_history_strided(const climber_config *cfg, const float *tau_layer, const void *q,
                         const void *k, const void *v, int64_t ld, const int32_t *scen,
                         const int32_t *beh, climber_kv_cache *cache, int32_t layer, void *o,
                         int64_t ld_o, hipStream_t s, const climber_rel_bias *bias = nullptr);
int attn_sumi_strided(const climber_config *cfg, const float *tau_layer,
                      const climber_kv_cache *cache, int32_t layer, const void *q, const void *k,
                      const void *v, int64_t ld, const int32_t *cand_off, int32_t m_total,
                      int32_t m_max, const int32_t *cscen, const int32_t *cbeh, void *o,
                      int64_t ld_o, hipStream_t s, const climber_rel_bias *bias = nullptr);
// History attention over a cache layer whose keys and values are already in place (written by the
// fused projection's epilogue, see QkvToCache in gemm.h): bf16 path only.
int attn_history_cached(const climber_config *cfg, const float *tau_layer, const void *q, int64_t ld_q,
                        const int32_t *scen, const int32_t *beh, climber_kv_cache *cache, int32_t layer,
                        void *o, int64_t ld_o, hipStream_t s);
// Where that epilogue has to write: fills every field but which0 and returns true if the cache is
// bf16 and holds rows (the CLIMBER_QKV_VIA_ROWS flag makes it return false).
struct QkvToCache;
bool cache_direct_target(const climber_config *cfg, climber_kv_cache *cache, int32_t layer, QkvToCache *out);
int64_t cache_rows(const climber_kv_cache *c);
int check_stack_call(const climber_config *cfg, const climber_kv_cache *cache, int32_t layer);
// the same for a call that only uses layer 0 of the cache as scratch: the cache may have been created
// for any number of layers
int check_scratch_cache(const climber_config *cfg, const climber_kv_cache *cache);

}  // namespace climber
