// Kernels of the bit-wise gating fusion module (bgf.hip); internal.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace climber {

// fusion attention over the n_blocks rows of every candidate; d_head = 64
hipError_t launch_bgf_attention(const void *qkv, void *o, const int32_t *scen, const float *tau_scen, int n_scen,
                                int64_t m, int nb, int H, float qk_scale, hipStream_t s);
// Y = G (.) sigmoid(pre), score = <w_head, Y> + b_head
hipError_t launch_bgf_gate_head(const float *g, const void *pre, const float *w_head, float b_head, float *y,
                                float *score, int64_t m, int nd, hipStream_t s);
int bgf_max_blocks();

}  // namespace climber
