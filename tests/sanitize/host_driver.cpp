// Driver for running the host side of libclimber (argument validation, cache handle bookkeeping,
// workspace carving) under AddressSanitizer / UBSan without a GPU: every call here must return its
// error code (or a size) before anything would be launched.  Device pointers are fake, never
// dereferenced on the host.
#include <cstdint>
#include <cstdio>
#include <vector>

#include "../../include/climber.h"

int main()
{
    void *fake = (void *)0x7F0000000000ull;
    int bad = 0;
    climber_config c{};
    c.n_layers = 4, c.d_model = 512, c.n_heads = 8, c.d_head = 64, c.d_ffn = 2048, c.n_scen = 8, c.n_beh = 4;
    c.sub_len = 256, c.dtype = CLIMBER_BF16, c.flags = 0, c.qk_scale = 1.f, c.rms_eps = 1e-6f;
    std::vector<int32_t> pad(32, 1024), len(32, 1000);
    bad |= climber_kv_cache_bytes(&c, 32, pad.data()) == 0;
    bad |= climber_workspace_bytes(&c, 40960) == 0;
    bad |= climber_packed_weights_bytes(&c) == 0;
    bad |= climber_bgf_workspace_bytes(&c, 4, 256, 8192) == 0;
    bad |= climber_bgf_workspace_bytes(&c, 17, 256, 8192) != 0;
    climber_kv_cache *h = nullptr;
    // no device in this process: the descriptor copy fails, the handle is released again
    const int rc = climber_kv_cache_create(&c, 32, len.data(), pad.data(), fake, (size_t)1 << 40, &h);
    bad |= rc == CLIMBER_OK && h == nullptr;
    if (h) climber_kv_cache_destroy(h);
    pad[3] = 1000;  // not a multiple of 64
    bad |= climber_kv_cache_create(&c, 32, len.data(), pad.data(), fake, (size_t)1 << 40, &h) != CLIMBER_ERR_ALIGN;
    bad |= climber_attn_sumi(&c, (const float *)fake, nullptr, 0, fake, fake, fake, (const int32_t *)fake, 8, 8,
                             (const int32_t *)fake, (const int32_t *)fake, fake, nullptr) != CLIMBER_ERR_NULL;
    climber_rel_bias rb{};
    bad |= climber_attn_sumi_bias(&c, (const float *)fake, nullptr, 0, fake, fake, fake, (const int32_t *)fake, 8, 8,
                                  (const int32_t *)fake, (const int32_t *)fake, fake, &rb, nullptr) != CLIMBER_ERR_NULL;
    climber_layer_weights lw{fake, fake, fake, fake, fake, fake};
    std::vector<climber_layer_weights> layers(4, lw);
    climber_weights w{4, layers.data(), nullptr};
    bad |= climber_pack_weights(&c, &w, fake, 16, nullptr) != CLIMBER_ERR_BUFSIZE;
    bad |= climber_sumi_score(&c, &w, (const float *)fake, nullptr, fake, (const int32_t *)fake, 8, 8,
                              (const int32_t *)fake, (const int32_t *)fake, (float *)fake, fake, 1 << 20, nullptr) !=
           CLIMBER_ERR_NULL;
    bad |= climber_sumi_score_static(&c, &w, (const float *)fake, nullptr, fake, (const int32_t *)fake, 8, 8,
                                     (const int32_t *)fake, (const int32_t *)fake, (float *)fake, nullptr) !=
           CLIMBER_ERR_NULL;
    climber_bgf_weights bw{};
    bw.n_blocks = 4, bw.d_gate = 256;
    bad |= climber_bgf_score(&c, &bw, (const float *)fake, (const int32_t *)fake, 8, nullptr, (float *)fake, fake, 1 << 20,
                             nullptr) != CLIMBER_ERR_NULL;
    for (int code = 0; code > -10; --code) bad |= climber_strerror(code) == nullptr;
    std::printf("host layer under sanitizers: bad=%d\n", bad);
    return bad;
}
