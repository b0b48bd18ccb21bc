"""MI355X-native Climber serving hot path: thin Python binding over libclimber.so.

The binding marshals arguments only; every step of the path runs in the HIP kernels of the
library.  There is no CPU fallback: using any compute entry point without the built library (or
without a GPU) raises.
"""
from .climber import (BAD_BEH, BAD_M_MAX, BAD_OFFSETS, BAD_SCEN, BAD_TAU, BF16, F32, HIST_CAUSAL, HIST_TWO_KERNEL, QKV_VIA_ROWS, MODE_CANDIDATE, MODE_HISTORY, ClimberError, Config, KVCache,
                      LayerWeights, STATIC_SCRATCH_BYTES, climber_attn_history, climber_attn_history_bias, climber_bgf_score, climber_bgf_workspace_bytes, BgfWeights, climber_attn_sumi, climber_attn_sumi_bias, climber_check_inputs, RelBias, rel_bias,
                      climber_history_encode, climber_kv_cache_bytes, climber_kv_cache_create,
                      climber_kv_cache_destroy, climber_kv_cache_rows, climber_layer_forward, climber_pack_weights,
                      climber_packed_weights_bytes,
                      climber_strerror, climber_sumi_forward, climber_sumi_score, climber_sumi_score_static, climber_workspace_bytes, library_path,
                      load_library)

__all__ = [n for n in dir() if not n.startswith("_")]
