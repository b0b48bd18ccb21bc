// Host side of libclimber.so: argument validation, the KV-cache handle and the dispatch of the
// C ABI declared in include/climber.h onto the HIP kernels.  Everything is validated before the
// first launch; nothing here allocates device memory.
#include "../../include/climber.h"

#include <algorithm>
#include <cmath>
#include <new>
#include <numeric>
#include <vector>

#include "internal.h"
#include "stack.h"
#include "gemm.h"

using namespace climber;

struct climber_kv_cache {
    climber_config cfg;
    int32_t B;
    std::vector<int32_t> hist_len, hist_pad, tok_off, order;
    uint8_t *dev;
    size_t bytes, header_bytes, layer_bytes;
    int32_t max_pad, max_len;
    int32_t uni_len, uni_pad;  // >= 0 when all users share one valid / padded length
    int64_t rows;
};

namespace {

size_t elem_size(int dtype) { return dtype == CLIMBER_BF16 ? 2 : 4; }
size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
bool aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }

int check_config(const climber_config *c)
{
    if (!c) return CLIMBER_ERR_NULL;
    if (c->n_layers < 1 || c->n_heads < 1 || c->d_head < 1 || c->n_scen < 1 || c->n_beh < 1 ||
        c->sub_len < 0 || c->d_model != c->n_heads * c->d_head)
        return CLIMBER_ERR_SHAPE;
    if (c->dtype != CLIMBER_F32 && c->dtype != CLIMBER_BF16) return CLIMBER_ERR_SHAPE;
    if (!(c->qk_scale > 0.f) || !std::isfinite(c->qk_scale)) return CLIMBER_ERR_TAU;
    if (c->flags & ~(CLIMBER_HIST_CAUSAL | CLIMBER_HIST_TWO_KERNEL | CLIMBER_QKV_VIA_ROWS)) return CLIMBER_ERR_SHAPE;
    if (c->dtype == CLIMBER_BF16) {
        if (c->d_head != kDHead) return CLIMBER_ERR_UNSUPPORTED;
        if (c->sub_len % 128 != 0) return CLIMBER_ERR_ALIGN;
    } else if (c->d_head > 256) {
        return CLIMBER_ERR_UNSUPPORTED;
    }
    return CLIMBER_OK;
}

// padded lengths: > 0, multiple of the path's padding unit; returns total rows or an error
int64_t check_padded(const climber_config *c, int32_t B, const int32_t *pad)
{
    if (B < 1) return CLIMBER_ERR_SHAPE;
    int64_t rows = 0;
    for (int b = 0; b < B; ++b) {
        if (pad[b] < 0) return CLIMBER_ERR_RANGE;
        if (c->dtype == CLIMBER_BF16 && pad[b] % 64 != 0) return CLIMBER_ERR_ALIGN;
        rows += pad[b];
    }
    if (rows * (int64_t)c->d_model >= (int64_t)1 << 31) return CLIMBER_ERR_RANGE;
    return rows;
}

// descriptor at the head of the device buffer: hist_len[B], tok_off[B+1], order[B] and, on the bf16
// path (padded lengths are multiples of 64), the user of every group of 64 padded rows
size_t header_bytes(const climber_config *c, int32_t B, int64_t rows)
{
    const size_t seg = c->dtype == CLIMBER_BF16 ? (size_t)(rows / 64) : 0;
    return round_up(((size_t)(3 * B + 1) + seg) * sizeof(int32_t), 256);
}

bool same_config(const climber_config &a, const climber_config &b)
{
    return a.n_layers == b.n_layers && a.d_model == b.d_model && a.n_heads == b.n_heads &&
           a.d_head == b.d_head && a.sub_len == b.sub_len && a.dtype == b.dtype;
}

CacheView view_of(const climber_kv_cache *k, int layer)
{
    CacheView v;
    const int32_t *hd = (const int32_t *)k->dev;
    v.hist_len = hd;
    v.tok_off = hd + k->B;
    v.order = hd + 2 * k->B + 1;
    v.seg = hd + 3 * k->B + 1;
    v.layer_base = k->dev + k->header_bytes + (size_t)layer * k->layer_bytes;
    v.B = k->B;
    return v;
}

int rt(hipError_t e) { return e == hipSuccess ? CLIMBER_OK : CLIMBER_ERR_RUNTIME; }

AttnArgs base_args(const climber_config *cfg, const climber_kv_cache *cache, int layer,
                   const float *tau)
{
    AttnArgs a{};
    a.cache = view_of(cache, layer);
    a.tau = tau;
    a.H = cfg->n_heads;
    a.d_head = cfg->d_head;
    a.n_scen = cfg->n_scen;
    a.n_beh = cfg->n_beh;
    a.sub_len = cfg->sub_len;
    a.causal = (cfg->flags & CLIMBER_HIST_CAUSAL) ? 1 : 0;
    a.qk_scale = cfg->qk_scale;
    a.max_hist_len = cache->max_len;
    a.uni_len = cache->uni_len;
    a.uni_pad = cache->uni_pad;
    a.uni_cand = -1;
    return a;
}

int check_cache_use(const climber_config *cfg, const climber_kv_cache *cache, int32_t layer)
{
    if (!cache) return CLIMBER_ERR_NULL;
    if (!same_config(*cfg, cache->cfg)) return CLIMBER_ERR_SHAPE;
    if (layer < 0 || layer >= cache->cfg.n_layers) return CLIMBER_ERR_RANGE;
    return CLIMBER_OK;
}

}  // namespace

// ---- internal entry points used by the stack driver (stack.hip) ---------------------------------
namespace climber {

int attn_history_strided(const climber_config *cfg, const float *tau_layer, const void *q,
                         const void *k, const void *v, int64_t ld, const int32_t *scen,
                         const int32_t *beh, climber_kv_cache *cache, int32_t layer, void *o,
                         int64_t ld_o, hipStream_t s, const climber_rel_bias *bias)
{
    const CacheView cv = view_of(cache, layer);
    if (cache->rows == 0) return CLIMBER_OK;
    // short subsequences, bf16: one kernel writes the cache and attends (K/V rows read once)
    const bool fused = cfg->dtype == CLIMBER_BF16 && o && !bias && !(cfg->flags & CLIMBER_HIST_TWO_KERNEL) &&
                       hist_fused_supported(cfg->sub_len, (cfg->flags & CLIMBER_HIST_CAUSAL) != 0);
    if (fused) {
    } else if (cfg->dtype == CLIMBER_BF16) {
        int e = rt(launch_kv_write_bf16(cv, k, v, ld, cfg->n_heads, cache->max_pad, s));
        if (e) return e;
    } else {
        int e = rt(launch_kv_write_f32(cv, k, v, ld, cfg->n_heads, cfg->d_head, cache->rows, s));
        if (e) return e;
    }
    if (!o) return CLIMBER_OK;
    AttnArgs a = base_args(cfg, cache, layer, tau_layer);
    a.q = q;
    a.k_self = k;  // a history row's own key seeds its softmax reference
    a.v_self = v;
    a.ld_q = ld;
    a.ld_kv = ld;
    a.scen = scen;
    a.beh = beh;
    a.o = o;
    a.ld_o = ld_o;
    a.max_rows_per_user = cache->max_pad;
    a.total_q_rows = cache->rows;
    if (bias) a.bias = BiasArgs{bias->pos_table, bias->time_table, bias->hist_pos, bias->hist_ts, bias->hist_pos,
                                bias->hist_ts, bias->n_pos, bias->n_time};
    if (fused) return rt(launch_hist_fused_bf16(a, s));
    if (cfg->dtype == CLIMBER_BF16) return rt(launch_attn_hist_bf16(a, s));
    return rt(launch_attn_f32(a, false, cache->rows, s));
}

int attn_history_cached(const climber_config *cfg, const float *tau_layer, const void *q, int64_t ld_q,
                        const int32_t *scen, const int32_t *beh, climber_kv_cache *cache, int32_t layer,
                        void *o, int64_t ld_o, hipStream_t s)
{
    if (cfg->dtype != CLIMBER_BF16) return CLIMBER_ERR_UNSUPPORTED;
    if (cache->rows == 0) return CLIMBER_OK;
    AttnArgs a = base_args(cfg, cache, layer, tau_layer);
    a.q = q;
    a.k_self = nullptr;  // the history pass of the tiled kernel reads keys and values from the cache only
    a.v_self = nullptr;
    a.ld_q = ld_q;
    a.ld_kv = ld_q;
    a.scen = scen;
    a.beh = beh;
    a.o = o;
    a.ld_o = ld_o;
    a.max_rows_per_user = cache->max_pad;
    a.total_q_rows = cache->rows;
    return rt(launch_attn_hist_bf16(a, s));
}

bool cache_direct_target(const climber_config *cfg, climber_kv_cache *cache, int32_t layer, QkvToCache *out)
{
    if ((cfg->flags & CLIMBER_QKV_VIA_ROWS) || cfg->dtype != CLIMBER_BF16 || cache->rows == 0) return false;
    const CacheView cv = view_of(cache, layer);
    out->layer_base = cv.layer_base;
    out->H = cfg->n_heads;
    out->l_valid = cache->uni_pad > 0 ? cache->uni_len : 0;
    out->l_pad = cache->uni_pad > 0 ? cache->uni_pad : 0;   // 0: per-user geometry from the tables
    out->d = cfg->d_model;
    out->which0 = 0;
    out->seg = cv.seg;
    out->tok_off = cv.tok_off;
    out->hist_len = cv.hist_len;
    out->rows = cache->rows;
    return true;
}

int attn_sumi_strided(const climber_config *cfg, const float *tau_layer,
                      const climber_kv_cache *cache, int32_t layer, const void *q, const void *k,
                      const void *v, int64_t ld, const int32_t *cand_off, int32_t m_total,
                      int32_t m_max, const int32_t *cscen, const int32_t *cbeh, void *o,
                      int64_t ld_o, hipStream_t s, const climber_rel_bias *bias)
{
    if (m_total == 0) return CLIMBER_OK;
    AttnArgs a = base_args(cfg, cache, layer, tau_layer);
    a.q = q;
    a.k_self = k;
    a.v_self = v;
    a.ld_q = ld;
    a.ld_kv = ld;
    a.scen = cscen;
    a.beh = cbeh;
    a.cand_off = cand_off;
    a.o = o;
    a.ld_o = ld_o;
    a.max_rows_per_user = m_max;
    a.total_q_rows = m_total;
    // m_max >= every user's count and the counts sum to m_total: equality means all are m_max
    if ((int64_t)m_max * cache->B == (int64_t)m_total) a.uni_cand = m_max;
    if (bias) a.bias = BiasArgs{bias->pos_table, bias->time_table, bias->hist_pos, bias->hist_ts, bias->cand_pos,
                                bias->cand_ts, bias->n_pos, bias->n_time};
    if (cfg->dtype == CLIMBER_BF16) return rt(launch_attn_sumi_bf16(a, s));
    return rt(launch_attn_f32(a, true, cache->rows, s));
}

int64_t cache_rows(const climber_kv_cache *c) { return c->rows; }

int check_stack_call(const climber_config *cfg, const climber_kv_cache *cache, int32_t layer)
{
    int e = check_config(cfg);
    if (e) return e;
    return check_cache_use(cfg, cache, layer);
}

int check_scratch_cache(const climber_config *cfg, const climber_kv_cache *cache)
{
    int e = check_config(cfg);
    if (e) return e;
    if (!cache) return CLIMBER_ERR_NULL;
    climber_config one = cache->cfg;
    one.n_layers = cfg->n_layers;
    return same_config(*cfg, one) ? CLIMBER_OK : CLIMBER_ERR_SHAPE;
}

}  // namespace climber

// ---- C ABI ------------------------------------------------------------------------------------
extern "C" {

const char *climber_strerror(int code)
{
    switch (code) {
    case CLIMBER_OK: return "ok";
    case CLIMBER_ERR_NULL: return "a required pointer is NULL";
    case CLIMBER_ERR_SHAPE: return "a size is non-positive or inconsistent";
    case CLIMBER_ERR_ALIGN: return "a padding, multiple-of or alignment rule is violated";
    case CLIMBER_ERR_RANGE: return "a layer index, length or offset is out of range";
    case CLIMBER_ERR_TAU: return "qk_scale or rms_eps is not finite and positive";
    case CLIMBER_ERR_BUFSIZE: return "a caller-provided buffer is too small";
    case CLIMBER_ERR_UNSUPPORTED: return "not supported by the selected precision path";
    case CLIMBER_ERR_RUNTIME: return "a HIP runtime call failed";
    default: return "unknown error code";
    }
}

size_t climber_kv_cache_bytes(const climber_config *cfg, int32_t B, const int32_t *hist_len_padded)
{
    if (check_config(cfg) != CLIMBER_OK || !hist_len_padded) return 0;
    const int64_t rows = check_padded(cfg, B, hist_len_padded);
    if (rows < 0) return 0;
    return header_bytes(cfg, B, rows) +
           (size_t)cfg->n_layers * 2 * (size_t)rows * cfg->d_model * elem_size(cfg->dtype);
}

int climber_kv_cache_create(const climber_config *cfg, int32_t B, const int32_t *hist_len,
                            const int32_t *hist_len_padded, void *dev_buf, size_t bytes,
                            climber_kv_cache **out)
{
    if (out) *out = nullptr;
    int e = check_config(cfg);
    if (e) return e;
    if (!hist_len || !hist_len_padded || !dev_buf || !out) return CLIMBER_ERR_NULL;
    const int64_t rows = check_padded(cfg, B, hist_len_padded);
    if (rows < 0) return (int)rows;
    int32_t max_len = 0, max_pad = 0;
    for (int b = 0; b < B; ++b) {
        if (hist_len[b] < 0 || hist_len[b] > hist_len_padded[b]) return CLIMBER_ERR_RANGE;
        max_len = std::max(max_len, hist_len[b]);
        max_pad = std::max(max_pad, hist_len_padded[b]);
    }
    if (cfg->dtype == CLIMBER_F32 && (size_t)max_len > attn_f32_max_keys())
        return CLIMBER_ERR_UNSUPPORTED;
    if (!aligned(dev_buf, 256)) return CLIMBER_ERR_ALIGN;
    const size_t need = climber_kv_cache_bytes(cfg, B, hist_len_padded);
    if (bytes < need) return CLIMBER_ERR_BUFSIZE;

    climber_kv_cache *k = new (std::nothrow) climber_kv_cache();
    if (!k) return CLIMBER_ERR_RUNTIME;
    k->cfg = *cfg;
    k->B = B;
    k->hist_len.assign(hist_len, hist_len + B);
    k->hist_pad.assign(hist_len_padded, hist_len_padded + B);
    k->tok_off.assign(B + 1, 0);
    for (int b = 0; b < B; ++b) k->tok_off[b + 1] = k->tok_off[b] + hist_len_padded[b];
    k->order.resize(B);
    std::iota(k->order.begin(), k->order.end(), 0);
    std::stable_sort(k->order.begin(), k->order.end(),
                     [&](int a, int b) { return k->hist_len[a] > k->hist_len[b]; });
    k->dev = (uint8_t *)dev_buf;
    k->bytes = bytes;
    k->header_bytes = header_bytes(cfg, B, rows);
    k->layer_bytes = 2 * (size_t)rows * cfg->d_model * elem_size(cfg->dtype);
    k->max_pad = max_pad;
    k->max_len = max_len;
    bool uni = true;
    for (int b = 1; b < B; ++b)
        uni = uni && hist_len[b] == hist_len[0] && hist_len_padded[b] == hist_len_padded[0];
    k->uni_len = uni ? hist_len[0] : -1;
    k->uni_pad = uni ? hist_len_padded[0] : -1;
    k->rows = rows;

    std::vector<int32_t> hd;
    hd.insert(hd.end(), k->hist_len.begin(), k->hist_len.end());
    hd.insert(hd.end(), k->tok_off.begin(), k->tok_off.end());
    hd.insert(hd.end(), k->order.begin(), k->order.end());
    if (cfg->dtype == CLIMBER_BF16)
        for (int b = 0; b < B; ++b) hd.insert(hd.end(), (size_t)(hist_len_padded[b] / 64), b);
    if (hipMemcpy(dev_buf, hd.data(), hd.size() * sizeof(int32_t), hipMemcpyHostToDevice) !=
        hipSuccess) {
        (void)hipGetLastError();
        delete k;
        return CLIMBER_ERR_RUNTIME;
    }
    *out = k;
    return CLIMBER_OK;
}

int climber_kv_cache_destroy(climber_kv_cache *cache)
{
    delete cache;
    return CLIMBER_OK;
}

int64_t climber_kv_cache_rows(const climber_kv_cache *cache)
{
    return cache ? cache->rows : (int64_t)CLIMBER_ERR_NULL;
}

static int check_bias(const climber_rel_bias *b, bool sumi)
{
    if (!b || !b->pos_table || !b->time_table || !b->hist_pos || !b->hist_ts) return CLIMBER_ERR_NULL;
    if (sumi && (!b->cand_pos || !b->cand_ts)) return CLIMBER_ERR_NULL;
    if (b->n_pos < 1 || b->n_pos % 2 == 0 || b->n_time < 1) return CLIMBER_ERR_SHAPE;
    if (!aligned(b->hist_pos, 16) || !aligned(b->hist_ts, 16)) return CLIMBER_ERR_ALIGN;
    return CLIMBER_OK;
}

static int attn_history_call(const climber_config *cfg, const float *tau_layer, const void *q,
                             const void *k, const void *v, const int32_t *scen, const int32_t *beh,
                             climber_kv_cache *cache, int32_t layer, void *o_hist,
                             const climber_rel_bias *bias, void *stream)
{
    int e = check_config(cfg);
    if (e) return e;
    e = check_cache_use(cfg, cache, layer);
    if (e) return e;
    if (!k || !v) return CLIMBER_ERR_NULL;
    if (o_hist && (!q || !scen || !beh || !tau_layer)) return CLIMBER_ERR_NULL;
    if (!aligned(k, 16) || !aligned(v, 16) || !aligned(q, 16) || !aligned(o_hist, 16))
        return CLIMBER_ERR_ALIGN;
    return attn_history_strided(cfg, tau_layer, q, k, v, cfg->d_model, scen, beh, cache, layer,
                                o_hist, cfg->d_model, (hipStream_t)stream, bias);
}

int climber_attn_history(const climber_config *cfg, const float *tau_layer, const void *q,
                         const void *k, const void *v, const int32_t *scen, const int32_t *beh,
                         climber_kv_cache *cache, int32_t layer, void *o_hist, void *stream)
{
    return attn_history_call(cfg, tau_layer, q, k, v, scen, beh, cache, layer, o_hist, nullptr, stream);
}

int climber_attn_history_bias(const climber_config *cfg, const float *tau_layer, const void *q,
                              const void *k, const void *v, const int32_t *scen, const int32_t *beh,
                              climber_kv_cache *cache, int32_t layer, void *o_hist,
                              const climber_rel_bias *bias, void *stream)
{
    const int e = check_bias(bias, false);
    if (e) return e;
    return attn_history_call(cfg, tau_layer, q, k, v, scen, beh, cache, layer, o_hist, bias, stream);
}

static int attn_sumi_call(const climber_config *cfg, const float *tau_layer,
                          const climber_kv_cache *cache, int32_t layer, const void *q_c,
                          const void *k_c, const void *v_c, const int32_t *cand_off, int32_t m_total,
                          int32_t m_max, const int32_t *cand_scen, const int32_t *cand_beh, void *o_c,
                          const climber_rel_bias *bias, void *stream)
{
    int e = check_config(cfg);
    if (e) return e;
    e = check_cache_use(cfg, cache, layer);
    if (e) return e;
    if (m_total < 0 || m_max < 0 || m_max > m_total) return CLIMBER_ERR_SHAPE;
    if ((int64_t)m_total * cfg->d_model >= (int64_t)1 << 31) return CLIMBER_ERR_RANGE;
    if (m_total > 0 && m_max == 0) return CLIMBER_ERR_SHAPE;
    if (!tau_layer || !cand_off) return CLIMBER_ERR_NULL;
    if (m_total == 0) return CLIMBER_OK;  // no candidates: the per-candidate arrays are empty, their pointers free
    if (!q_c || !k_c || !v_c || !cand_scen || !cand_beh || !o_c) return CLIMBER_ERR_NULL;
    if (!aligned(q_c, 16) || !aligned(k_c, 16) || !aligned(v_c, 16) || !aligned(o_c, 16))
        return CLIMBER_ERR_ALIGN;
    return attn_sumi_strided(cfg, tau_layer, cache, layer, q_c, k_c, v_c, cfg->d_model, cand_off,
                             m_total, m_max, cand_scen, cand_beh, o_c, cfg->d_model,
                             (hipStream_t)stream, bias);
}

int climber_attn_sumi(const climber_config *cfg, const float *tau_layer,
                      const climber_kv_cache *cache, int32_t layer, const void *q_c,
                      const void *k_c, const void *v_c, const int32_t *cand_off, int32_t m_total,
                      int32_t m_max, const int32_t *cand_scen, const int32_t *cand_beh, void *o_c,
                      void *stream)
{
    return attn_sumi_call(cfg, tau_layer, cache, layer, q_c, k_c, v_c, cand_off, m_total, m_max, cand_scen,
                          cand_beh, o_c, nullptr, stream);
}

int climber_attn_sumi_bias(const climber_config *cfg, const float *tau_layer,
                           const climber_kv_cache *cache, int32_t layer, const void *q_c,
                           const void *k_c, const void *v_c, const int32_t *cand_off,
                           int32_t m_total, int32_t m_max, const int32_t *cand_scen,
                           const int32_t *cand_beh, void *o_c, const climber_rel_bias *bias,
                           void *stream)
{
    const int e = check_bias(bias, true);
    if (e) return e;
    return attn_sumi_call(cfg, tau_layer, cache, layer, q_c, k_c, v_c, cand_off, m_total, m_max, cand_scen,
                          cand_beh, o_c, bias, stream);
}

int climber_check_inputs(const climber_config *cfg, const float *tau_layer, const int32_t *scen,
                         const int32_t *beh, const climber_kv_cache *cache, int32_t m_total,
                         const int32_t *cand_off, int32_t B_cand, int32_t m_max, int32_t *status,
                         void *stream)
{
    int e = check_config(cfg);
    if (e) return e;
    if (!tau_layer || !scen || !beh || !status) return CLIMBER_ERR_NULL;
    if (cache) {
        if (!same_config(*cfg, cache->cfg)) return CLIMBER_ERR_SHAPE;
        const CacheView cv = view_of(cache, 0);
        return rt(launch_check_inputs(tau_layer, scen, beh, cache->rows, cv.hist_len, cv.tok_off, nullptr,
                                      cache->B, cfg->n_scen, cfg->n_beh, 0, status, (hipStream_t)stream));
    }
    if (m_total < 0 || (cand_off && B_cand < 1)) return CLIMBER_ERR_SHAPE;
    return rt(launch_check_inputs(tau_layer, scen, beh, m_total, nullptr, nullptr, cand_off, B_cand,
                                  cfg->n_scen, cfg->n_beh, m_max, status, (hipStream_t)stream));
}

}  // extern "C"
