// Layer-stack driver: the serving flow of Climber (arXiv 2502.09888, Sec. 3.2) over the full
// layers -- history encode (fills every layer of the KV cache) and candidate scoring against it.
// Layer composition (the paper leaves f_QKV / f_FFN of Eq. (3) open; this build fixes it):
//   qkv = RMSNorm(x; g1) Wqkv;  o = attention;  h = x + o Wo;  y = h + GELU(RMSNorm(h; g2) W1) W2
// The residual stream is fp32, GEMM operands are bf16, accumulation is fp32.  RMSNorm never runs
// as a kernel of its own: RMSNorm(x; g) W = r * (x (g (.) W)) with r = 1/sqrt(mean(x^2) + eps) per
// row, so the gains are folded into the weight rows when the weights are repacked, the projection
// that produces x also emits its bf16 copy and the row sums of squares, and the projection that
// consumes it scales its output rows by r.
#include "stack.h"

#include <algorithm>
#include <cmath>
#include <mutex>

#include "bgf.h"
#include "gemm.h"

using namespace climber;

namespace {

size_t up256(size_t x) { return (x + 255) / 256 * 256; }

struct Workspace {
    float *x32;     // [rows][d]   residual stream of encode / score
    float *h32;     // [rows][d]   post-attention residual
    uint8_t *xb;    // [rows][d]   bf16 copy of the rows the next projection normalises
    float *ss;      // [rows][d/64] partial sums of squares of those rows
    uint8_t *qkv;   // [rows][3d]  bf16 fused projection output
    uint8_t *o;     // [rows][d]   bf16 attention output
    uint8_t *u;     // bf16 FFN hidden, tiled layout (gemm.h), rows rounded up to 16
    uint8_t *wpack; // packed weights of every layer: [layer]{wqkv, wo, w1, w2}
    size_t wlayer;  // bytes of one layer's packed weights
    size_t total;
};

struct PackedLayer { const uint8_t *wqkv, *wo, *w1, *w2; };

Workspace carve(const climber_config *c, int64_t rows, void *base, bool with_weights = true)
{
    const size_t d = c->d_model, F = c->d_ffn, n = (size_t)rows;
    uint8_t *p = (uint8_t *)base;
    size_t off = 0;
    auto take = [&](size_t bytes) { uint8_t *q = p + off; off += up256(bytes); return q; };
    Workspace w;
    w.x32 = (float *)take(n * d * 4);
    w.h32 = (float *)take(n * d * 4);
    w.xb = take(n * d * 2);
    w.ss = (float *)take(n * (d / 64) * 4);
    w.qkv = take(n * 3 * d * 2);
    w.o = take(n * d * 2);
    w.u = take((n + 15) / 16 * 16 * F * 2);
    w.wlayer = up256((4 * d * d + 2 * d * F) * 2);
    w.wpack = with_weights ? take(w.wlayer * (size_t)std::max(c->n_layers, 1)) : nullptr;
    w.total = off;
    return w;
}

PackedLayer packed_layer(const climber_config *c, const Workspace &ws, int slot)
{
    const size_t d = c->d_model, F = c->d_ffn;
    const uint8_t *b = ws.wpack + ws.wlayer * (size_t)slot;
    return PackedLayer{b, b + 3 * d * d * 2, b + 4 * d * d * 2, b + (4 * d * d + d * F) * 2};
}

int check_stack_config(const climber_config *c)
{
    if (!c) return CLIMBER_ERR_NULL;
    if (c->dtype != CLIMBER_BF16) return CLIMBER_ERR_UNSUPPORTED;
    if (c->d_ffn < 1) return CLIMBER_ERR_SHAPE;
    if (c->d_model % 128 != 0 || c->d_ffn % 128 != 0) return CLIMBER_ERR_UNSUPPORTED;
    if (!(c->rms_eps > 0.f) || !std::isfinite(c->rms_eps)) return CLIMBER_ERR_TAU;
    return CLIMBER_OK;
}

int rt(hipError_t e) { return e == hipSuccess ? CLIMBER_OK : CLIMBER_ERR_RUNTIME; }

#define TRY(x)            \
    do {                  \
        int e_ = (x);     \
        if (e_) return e_; \
    } while (0)

// MFMA fragment order for the weights of layers [0, n) into slots [0, n) of the workspace: one
// launch per four layers
int pack_layers(const climber_config *cfg, const climber_layer_weights *layers, int n,
                const Workspace &ws, hipStream_t s)
{
    const int d = cfg->d_model, F = cfg->d_ffn;
    PackJobs jobs;
    jobs.n = 0;
    for (int l = 0; l < n; ++l) {
        const PackedLayer pl = packed_layer(cfg, ws, l);
        const void *src[4] = {layers[l].wqkv, layers[l].wo, layers[l].w1, layers[l].w2};
        const void *gain[4] = {layers[l].g1, nullptr, layers[l].g2, nullptr};
        const uint8_t *dst[4] = {pl.wqkv, pl.wo, pl.w1, pl.w2};
        const int K[4] = {d, d, d, F}, N[4] = {3 * d, d, F, d};
        for (int i = 0; i < 4; ++i) {
            jobs.w[jobs.n] = src[i];
            jobs.gain[jobs.n] = gain[i];
            jobs.packed[jobs.n] = const_cast<uint8_t *>(dst[i]);
            jobs.K[jobs.n] = K[i];
            jobs.N[jobs.n] = N[i];
            ++jobs.n;
        }
        if (jobs.n == kMaxPackJobs || l + 1 == n) {
            TRY(rt(pack_weights(jobs, s)));
            jobs.n = 0;
        }
    }
    return CLIMBER_OK;
}

// one layer on `rows` rows.  x_in: fp32 rows (the residual stream); xb_in / ws.ss: their bf16 copy and
// row sums of squares (from the previous layer's last projection or from a row_prep kernel).
// norm_out: also emit the bf16 copy and sums of squares of x_out (the next layer needs them).
int run_layer(const climber_config *cfg, const PackedLayer &pw, const float *tau_layer, int32_t layer,
              int32_t mode, climber_kv_cache *cache, const float *x_in, const void *xb_in, float *x_out,
              bool norm_out, const int32_t *scen, const int32_t *beh, const int32_t *cand_off,
              int32_t m_total, int32_t m_max, int64_t rows, const Workspace &ws, hipStream_t s)
{
    const int d = cfg->d_model, F = cfg->d_ffn, M = (int)rows;
    const RowNormIn nin{ws.ss, d / 64, 1.f / (float)d, cfg->rms_eps}, no_in{nullptr, 0, 0.f, 0.f};
    const RowNormOut nout{ws.ss, ws.xb, d}, no_out{nullptr, nullptr, 0};
    QkvToCache qc;
    if (mode == CLIMBER_MODE_HISTORY && cache_direct_target(cfg, cache, layer, &qc)) {
        // the projection's epilogue writes keys and values into the cache as operand fragments; only
        // the query rows exist as rows (the last layer needs none at all)
        if (!x_out) {
            qc.which0 = 1;
            return rt(gemm_bf16(EPI_STORE_BF16, xb_in, d, pw.wqkv + (size_t)d * d * 2, M, 2 * d, d, ws.qkv, d,
                                nullptr, 0, nin, no_out, 0, s, &qc));
        }
        TRY(rt(gemm_bf16(EPI_STORE_BF16, xb_in, d, pw.wqkv, M, 3 * d, d, ws.qkv, d, nullptr, 0, nin, no_out, 0,
                         s, &qc)));
        TRY(attn_history_cached(cfg, tau_layer, ws.qkv, d, scen, beh, cache, layer, ws.o, d, s));
    } else {
        TRY(rt(gemm_bf16(EPI_STORE_BF16, xb_in, d, pw.wqkv, M, 3 * d, d, ws.qkv, 3 * d, nullptr, 0, nin,
                         no_out, 0, s)));
        const uint8_t *q = ws.qkv, *k = ws.qkv + (size_t)d * 2, *v = ws.qkv + (size_t)2 * d * 2;
        if (mode == CLIMBER_MODE_HISTORY) {
            TRY(attn_history_strided(cfg, tau_layer, q, k, v, 3 * d, scen, beh, cache, layer,
                                     x_out ? ws.o : nullptr, d, s));
            if (!x_out) return CLIMBER_OK;
        } else {
            TRY(attn_sumi_strided(cfg, tau_layer, cache, layer, q, k, v, 3 * d, cand_off, m_total, m_max,
                                  scen, beh, ws.o, d, s));
        }
    }
    TRY(rt(gemm_bf16(EPI_RESID_F32, ws.o, d, pw.wo, M, d, d, ws.h32, d, x_in, d, no_in, nout, 0, s)));
    TRY(rt(gemm_bf16(EPI_GELU_BF16, ws.xb, d, pw.w1, M, F, d, ws.u, F, nullptr, 0, nin, no_out, kTiledC, s)));
    TRY(rt(gemm_bf16(EPI_RESID_F32, ws.u, F, pw.w2, M, d, F, x_out, d, ws.h32, d, no_in,
                     norm_out ? nout : no_out, kTiledA, s)));
    return CLIMBER_OK;
}

int check_layer_weights(const climber_layer_weights *w)
{
    if (!w || !w->g1 || !w->wqkv || !w->wo || !w->g2 || !w->w1 || !w->w2) return CLIMBER_ERR_NULL;
    const void *ps[] = {w->g1, w->wqkv, w->wo, w->g2, w->w1, w->w2};
    for (const void *p : ps)
        if ((uintptr_t)p % 16 != 0) return CLIMBER_ERR_ALIGN;
    return CLIMBER_OK;
}

// weights of a whole-stack call: either prepacked (weights->packed) or per-layer pointers
int check_weights(const climber_config *cfg, const climber_weights *weights)
{
    if (!weights) return CLIMBER_ERR_NULL;
    if (weights->n_layers != cfg->n_layers) return CLIMBER_ERR_SHAPE;
    if (weights->packed) return (uintptr_t)weights->packed % 256 == 0 ? CLIMBER_OK : CLIMBER_ERR_ALIGN;
    if (!weights->layers) return CLIMBER_ERR_NULL;
    for (int l = 0; l < cfg->n_layers; ++l) TRY(check_layer_weights(&weights->layers[l]));
    return CLIMBER_OK;
}

// packed weights in place for the call: the caller's buffer, or the workspace's after one launch
int stage_weights(const climber_config *cfg, const climber_weights *weights, Workspace &ws, hipStream_t s)
{
    if (weights->packed) {
        ws.wpack = (uint8_t *)const_cast<void *>(weights->packed);
        return CLIMBER_OK;
    }
    return pack_layers(cfg, weights->layers, cfg->n_layers, ws, s);
}

int check_cand_args(const climber_config *cfg, const int32_t *cand_off, int32_t m_total, int32_t m_max)
{
    if (!cand_off) return CLIMBER_ERR_NULL;
    if (m_total < 0 || m_max < 0 || m_max > m_total || (m_total > 0 && m_max == 0))
        return CLIMBER_ERR_SHAPE;
    if ((int64_t)m_total * std::max(cfg->d_ffn, 3 * cfg->d_model) >= (int64_t)1 << 31)
        return CLIMBER_ERR_RANGE;
    return CLIMBER_OK;
}

int check_score_args(const climber_config *cfg, const climber_weights *weights, const float *tau,
                     const climber_kv_cache *cache, const void *x_cand, const int32_t *cand_off,
                     int32_t m_total, int32_t m_max, const int32_t *cand_scen, const int32_t *cand_beh,
                     const float *y_cand)
{
    TRY(check_stack_config(cfg));
    TRY(check_stack_call(cfg, cache, 0));
    if (!tau) return CLIMBER_ERR_NULL;
    TRY(check_weights(cfg, weights));
    TRY(check_cand_args(cfg, cand_off, m_total, m_max));
    if (m_total == 0) return CLIMBER_OK;  // no candidates: the per-candidate arrays are empty, their pointers free
    if (!x_cand || !cand_scen || !cand_beh || !y_cand) return CLIMBER_ERR_NULL;
    if ((uintptr_t)x_cand % 16 != 0 || (uintptr_t)y_cand % 16 != 0) return CLIMBER_ERR_ALIGN;
    return CLIMBER_OK;
}

// candidate rows through every layer against the cache; ws: carved scratch for m_total rows
int score_layers(const climber_config *cfg, const climber_weights *weights, const float *tau,
                 const climber_kv_cache *cache, const void *x_cand, const int32_t *cand_off,
                 int32_t m_total, int32_t m_max, const int32_t *cand_scen, const int32_t *cand_beh,
                 float *y_cand, Workspace &ws, hipStream_t s)
{
    if (m_total == 0) return CLIMBER_OK;
    TRY(stage_weights(cfg, weights, ws, s));
    TRY(rt(row_prep_bf16(x_cand, ws.x32, ws.ss, cfg->d_model / 64, m_total, cfg->d_model, s)));
    const size_t tl = (size_t)cfg->n_scen * cfg->n_beh;
    for (int l = 0; l < cfg->n_layers; ++l) {
        const bool last = l + 1 == cfg->n_layers;
        // the cache is only read in candidate mode
        TRY(run_layer(cfg, packed_layer(cfg, ws, l), tau + l * tl, l, CLIMBER_MODE_CANDIDATE,
                      const_cast<climber_kv_cache *>(cache), ws.x32, l == 0 ? x_cand : (const void *)ws.xb,
                      last ? y_cand : ws.x32, !last, cand_scen, cand_beh, cand_off, m_total, m_max,
                      m_total, ws, s));
    }
    return CLIMBER_OK;
}

// ---- scratch of the allocation-free scoring call ---------------------------------------------
// One array per device, part of the library's code object: it exists on every GPU the library is
// loaded on until the process ends.  Nothing in it has to start at zero (every region is written
// before it is read within a call).  In host code the array's name is only a handle for the
// symbol lookup; kernels are given the device address that lookup returned, one per device.
static __device__ __align__(256) unsigned char scratch[CLIMBER_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
uint8_t *scratch_ptr[kMaxDevices];  // device address of `scratch` on device i, once looked up

int static_scratch(uint8_t **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return CLIMBER_ERR_RUNTIME;
    }
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return CLIMBER_ERR_RUNTIME;
        }
        scratch_ptr[dev] = (uint8_t *)ptr;
    }
    *out = scratch_ptr[dev];
    return CLIMBER_OK;
}

}  // namespace

extern "C" {

size_t climber_workspace_bytes(const climber_config *cfg, int64_t max_rows)
{
    if (check_stack_config(cfg) != CLIMBER_OK || max_rows < 0) return 0;
    return carve(cfg, max_rows, nullptr).total;
}

size_t climber_packed_weights_bytes(const climber_config *cfg)
{
    if (check_stack_config(cfg) != CLIMBER_OK || cfg->n_layers < 1) return 0;
    return carve(cfg, 0, nullptr).wlayer * (size_t)cfg->n_layers;
}

int climber_pack_weights(const climber_config *cfg, const climber_weights *weights, void *packed,
                         size_t bytes, void *stream)
{
    TRY(check_stack_config(cfg));
    if (cfg->n_layers < 1) return CLIMBER_ERR_SHAPE;
    if (!weights || !weights->layers || !packed) return CLIMBER_ERR_NULL;
    if (weights->n_layers != cfg->n_layers) return CLIMBER_ERR_SHAPE;
    for (int l = 0; l < cfg->n_layers; ++l) TRY(check_layer_weights(&weights->layers[l]));
    if ((uintptr_t)packed % 256 != 0) return CLIMBER_ERR_ALIGN;
    if (bytes < climber_packed_weights_bytes(cfg)) return CLIMBER_ERR_BUFSIZE;
    Workspace ws = carve(cfg, 0, nullptr);
    ws.wpack = (uint8_t *)packed;
    return pack_layers(cfg, weights->layers, cfg->n_layers, ws, (hipStream_t)stream);
}

int climber_layer_forward(const climber_config *cfg, const climber_layer_weights *w,
                          const float *tau_layer, int32_t layer, int32_t mode,
                          climber_kv_cache *cache, const float *x_in, float *x_out,
                          const int32_t *scen, const int32_t *beh, const int32_t *cand_off,
                          int32_t m_total, int32_t m_max, void *workspace, size_t ws_bytes,
                          void *stream)
{
    TRY(check_stack_config(cfg));
    TRY(check_stack_call(cfg, cache, layer));
    TRY(check_layer_weights(w));
    if (mode != CLIMBER_MODE_HISTORY && mode != CLIMBER_MODE_CANDIDATE) return CLIMBER_ERR_SHAPE;
    if (!tau_layer || !x_in || !scen || !beh || !workspace) return CLIMBER_ERR_NULL;
    if (mode == CLIMBER_MODE_CANDIDATE) {
        if (!x_out) return CLIMBER_ERR_NULL;
        TRY(check_cand_args(cfg, cand_off, m_total, m_max));
    }
    const int64_t rows = mode == CLIMBER_MODE_HISTORY ? cache_rows(cache) : m_total;
    if (rows * (int64_t)std::max(cfg->d_ffn, 3 * cfg->d_model) >= (int64_t)1 << 31)
        return CLIMBER_ERR_RANGE;
    if ((uintptr_t)workspace % 256 != 0 || (uintptr_t)x_in % 16 != 0 || (uintptr_t)x_out % 16 != 0)
        return CLIMBER_ERR_ALIGN;
    const Workspace ws = carve(cfg, rows, workspace);
    if (ws_bytes < ws.total) return CLIMBER_ERR_BUFSIZE;
    if (rows == 0) return CLIMBER_OK;
    hipStream_t s = (hipStream_t)stream;
    TRY(pack_layers(cfg, w, 1, ws, s));
    TRY(rt(row_prep_f32(x_in, ws.xb, ws.ss, cfg->d_model / 64, rows, cfg->d_model, s)));
    return run_layer(cfg, packed_layer(cfg, ws, 0), tau_layer, layer, mode, cache, x_in, ws.xb, x_out,
                     false, scen, beh, cand_off, m_total, m_max, rows, ws, s);
}

int climber_history_encode(const climber_config *cfg, const climber_weights *weights,
                           const float *tau, const void *x_hist, const int32_t *scen,
                           const int32_t *beh, climber_kv_cache *cache, void *workspace,
                           size_t ws_bytes, void *stream)
{
    TRY(check_stack_config(cfg));
    TRY(check_stack_call(cfg, cache, 0));
    if (!tau || !x_hist || !scen || !beh || !workspace) return CLIMBER_ERR_NULL;
    TRY(check_weights(cfg, weights));
    const int64_t rows = cache_rows(cache);
    if (rows * (int64_t)std::max(cfg->d_ffn, 3 * cfg->d_model) >= (int64_t)1 << 31)
        return CLIMBER_ERR_RANGE;
    if ((uintptr_t)workspace % 256 != 0 || (uintptr_t)x_hist % 16 != 0) return CLIMBER_ERR_ALIGN;
    Workspace ws = carve(cfg, rows, workspace);
    if (ws_bytes < ws.total) return CLIMBER_ERR_BUFSIZE;
    if (rows == 0) return CLIMBER_OK;
    hipStream_t s = (hipStream_t)stream;
    TRY(stage_weights(cfg, weights, ws, s));
    TRY(rt(row_prep_bf16(x_hist, ws.x32, ws.ss, cfg->d_model / 64, rows, cfg->d_model, s)));
    const size_t tl = (size_t)cfg->n_scen * cfg->n_beh;
    for (int l = 0; l < cfg->n_layers; ++l) {
        const bool last = l + 1 == cfg->n_layers;  // nothing reads the last layer's history output
        TRY(run_layer(cfg, packed_layer(cfg, ws, l), tau + l * tl, l, CLIMBER_MODE_HISTORY, cache,
                      ws.x32, l == 0 ? x_hist : (const void *)ws.xb, last ? nullptr : ws.x32, !last, scen,
                      beh, nullptr, 0, 0, rows, ws, s));
    }
    return CLIMBER_OK;
}

// ---- bit-wise gating fusion (Eq. (4)) -------------------------------------------------------
// scratch = the stack's scratch for m * n_blocks rows and one layer (the fusion layer) + the packed
// gate weights
static size_t bgf_gate_bytes(const climber_config *cfg, int nb, int dg)
{
    return up256((size_t)2 * nb * cfg->d_model * dg * 2);
}

static int check_bgf(const climber_config *cfg, int32_t n_blocks, int32_t d_gate)
{
    TRY(check_stack_config(cfg));
    if (cfg->d_head != 64 || cfg->n_heads * 64 != cfg->d_model) return CLIMBER_ERR_UNSUPPORTED;
    if (n_blocks < 1 || n_blocks > bgf_max_blocks() || d_gate < 1) return CLIMBER_ERR_SHAPE;
    if (d_gate % 128 != 0 || d_gate > n_blocks * cfg->d_model) return CLIMBER_ERR_UNSUPPORTED;
    return CLIMBER_OK;
}

size_t climber_bgf_workspace_bytes(const climber_config *cfg, int32_t n_blocks, int32_t d_gate, int64_t m_total)
{
    if (check_bgf(cfg, n_blocks, d_gate) != CLIMBER_OK || m_total < 0) return 0;
    climber_config one = *cfg;
    one.n_layers = 1;
    return carve(&one, m_total * n_blocks, nullptr).total + bgf_gate_bytes(cfg, n_blocks, d_gate);
}

int climber_bgf_score(const climber_config *cfg, const climber_bgf_weights *w, const float *e,
                      const int32_t *cand_scen, int32_t m_total, float *y, float *score, void *workspace,
                      size_t ws_bytes, void *stream)
{
    if (!w) return CLIMBER_ERR_NULL;
    TRY(check_bgf(cfg, w->n_blocks, w->d_gate));
    TRY(check_layer_weights(&w->atl));
    if (!w->w_down || !w->w_up || !w->w_head || !w->tau_scen || !e || !cand_scen || !score || !workspace)
        return CLIMBER_ERR_NULL;
    if (m_total < 0) return CLIMBER_ERR_SHAPE;
    const int nb = w->n_blocks, dg = w->d_gate, d = cfg->d_model, F = cfg->d_ffn, nd = nb * d, np = d / 64;
    const int64_t R = (int64_t)m_total * nb;
    if (R * (int64_t)std::max(F, 3 * d) >= (int64_t)1 << 31) return CLIMBER_ERR_RANGE;
    if ((uintptr_t)workspace % 256 != 0 || (uintptr_t)e % 16 != 0 || (uintptr_t)y % 16 != 0 ||
        (uintptr_t)w->w_down % 16 != 0 || (uintptr_t)w->w_up % 16 != 0 || (uintptr_t)w->w_head % 16 != 0)
        return CLIMBER_ERR_ALIGN;
    climber_config one = *cfg;
    one.n_layers = 1;
    Workspace ws = carve(&one, R, workspace);
    uint8_t *gate_pack = (uint8_t *)workspace + ws.total;
    if (ws_bytes < ws.total + bgf_gate_bytes(cfg, nb, dg)) return CLIMBER_ERR_BUFSIZE;
    if (m_total == 0) return CLIMBER_OK;
    hipStream_t s = (hipStream_t)stream;
    // operand order for the fusion layer's weights (gains folded in) and the two gate projections
    TRY(pack_layers(&one, &w->atl, 1, ws, s));
    uint8_t *down_p = gate_pack, *up_p = gate_pack + (size_t)nd * dg * 2;
    {
        PackJobs jobs;
        jobs.n = 2;
        jobs.w[0] = w->w_down, jobs.gain[0] = nullptr, jobs.packed[0] = down_p, jobs.K[0] = nd, jobs.N[0] = dg;
        jobs.w[1] = w->w_up, jobs.gain[1] = nullptr, jobs.packed[1] = up_p, jobs.K[1] = dg, jobs.N[1] = nd;
        TRY(rt(pack_weights(jobs, s)));
    }
    const PackedLayer pw = packed_layer(&one, ws, 0);
    const RowNormIn nin{ws.ss, np, 1.f / (float)d, cfg->rms_eps}, no_in{nullptr, 0, 0.f, 0.f};
    const RowNormOut nout{ws.ss, ws.xb, d}, no_out{nullptr, nullptr, 0};
    // G = ATL(E) on the m * n_blocks rows: the layer of the stack with the fusion attention in the middle
    TRY(rt(row_prep_f32(e, ws.xb, ws.ss, np, R, d, s)));
    TRY(rt(gemm_bf16(EPI_STORE_BF16, ws.xb, d, pw.wqkv, (int)R, 3 * d, d, ws.qkv, 3 * d, nullptr, 0, nin, no_out, 0, s)));
    TRY(rt(launch_bgf_attention(ws.qkv, ws.o, cand_scen, w->tau_scen, cfg->n_scen, m_total, nb, cfg->n_heads,
                                cfg->qk_scale, s)));
    TRY(rt(gemm_bf16(EPI_RESID_F32, ws.o, d, pw.wo, (int)R, d, d, ws.h32, d, e, d, no_in, nout, 0, s)));
    TRY(rt(gemm_bf16(EPI_GELU_BF16, ws.xb, d, pw.w1, (int)R, F, d, ws.u, F, nullptr, 0, nin, no_out, kTiledC, s)));
    TRY(rt(gemm_bf16(EPI_RESID_F32, ws.u, F, pw.w2, (int)R, d, F, ws.x32, d, ws.h32, d, no_in, nout, kTiledA, s)));
    // f_gate on the flattened G (its bf16 copy, [m][n_blocks * d]): down, ReLU, up; then sigmoid,
    // Hadamard product and the head in one pass over G
    TRY(rt(gemm_bf16(EPI_RELU_BF16, ws.xb, nd, down_p, m_total, dg, nd, ws.o, dg, nullptr, 0, no_in, no_out, 0, s)));
    TRY(rt(gemm_bf16(EPI_STORE_BF16, ws.o, dg, up_p, m_total, nd, dg, ws.qkv, nd, nullptr, 0, no_in, no_out, 0, s)));
    return rt(launch_bgf_gate_head(ws.x32, ws.qkv, w->w_head, w->b_head, y, score, m_total, nd, s));
}

int climber_sumi_forward(const climber_config *cfg, const climber_weights *weights, const float *tau,
                         const void *x_hist, const int32_t *scen, const int32_t *beh, const void *x_cand,
                         const int32_t *cand_off, int32_t m_total, int32_t m_max,
                         const int32_t *cand_scen, const int32_t *cand_beh, climber_kv_cache *scratch_cache,
                         float *y_hist, float *y_cand, void *workspace, size_t ws_bytes, void *stream)
{
    TRY(check_stack_config(cfg));
    TRY(check_scratch_cache(cfg, scratch_cache));
    if (!tau || !x_hist || !scen || !beh || !workspace) return CLIMBER_ERR_NULL;
    // (no candidates: the per-candidate arrays are empty, their pointers free)
    if (m_total > 0 && (!x_cand || !cand_scen || !cand_beh || !y_cand)) return CLIMBER_ERR_NULL;
    TRY(check_weights(cfg, weights));
    TRY(check_cand_args(cfg, cand_off, m_total, m_max));
    const int64_t T = cache_rows(scratch_cache), R = T + m_total;
    if (R * (int64_t)std::max(cfg->d_ffn, 3 * cfg->d_model) >= (int64_t)1 << 31) return CLIMBER_ERR_RANGE;
    if ((uintptr_t)workspace % 256 != 0 || (uintptr_t)x_hist % 16 != 0 || (uintptr_t)x_cand % 16 != 0 ||
        (uintptr_t)y_cand % 16 != 0 || (uintptr_t)y_hist % 16 != 0)
        return CLIMBER_ERR_ALIGN;
    Workspace ws = carve(cfg, R, workspace);
    if (ws_bytes < ws.total) return CLIMBER_ERR_BUFSIZE;
    if (R == 0) return CLIMBER_OK;
    hipStream_t s = (hipStream_t)stream;
    const int d = cfg->d_model, F = cfg->d_ffn, np = d / 64;
    TRY(stage_weights(cfg, weights, ws, s));
    // rows [0, T): the padded history rows of the batch; rows [T, R): the candidates
    TRY(rt(row_prep_bf16(x_hist, ws.x32, ws.ss, np, T, d, s)));
    TRY(rt(row_prep_bf16(x_cand, ws.x32 + (size_t)T * d, ws.ss + (size_t)T * np, np, m_total, d, s)));
    if (T) TRY(rt(hipMemcpyAsync(ws.xb, x_hist, (size_t)T * d * 2, hipMemcpyDeviceToDevice, s)));
    if (m_total)
        TRY(rt(hipMemcpyAsync(ws.xb + (size_t)T * d * 2, x_cand, (size_t)m_total * d * 2, hipMemcpyDeviceToDevice, s)));
    const RowNormIn nin{ws.ss, np, 1.f / (float)d, cfg->rms_eps}, no_in{nullptr, 0, 0.f, 0.f};
    const RowNormOut no_out{nullptr, nullptr, 0};
    const size_t tl = (size_t)cfg->n_scen * cfg->n_beh;
    for (int l = 0; l < cfg->n_layers; ++l) {
        const bool last = l + 1 == cfg->n_layers;
        const PackedLayer pw = packed_layer(cfg, ws, l);
        const float *tau_l = tau + l * tl;
        const size_t crow = (size_t)T * 3 * d * 2;  // the candidates' part of the projection output
        const uint8_t *q = ws.qkv, *k = q + (size_t)d * 2, *v = q + (size_t)2 * d * 2;
        // the history's outputs of the last layer feed nothing unless the caller wants them
        const bool hist_out = !last || y_hist;
        QkvToCache qc;
        if (T > 0 && cache_direct_target(cfg, scratch_cache, 0, &qc)) {
            // history rows: the projection's epilogue writes keys and values into layer 0 of the scratch
            // cache as operand fragments and the queries as rows of d (none of them when nothing follows);
            // the candidates' rows get a projection launch of their own
            if (hist_out) {
                TRY(rt(gemm_bf16(EPI_STORE_BF16, ws.xb, d, pw.wqkv, (int)T, 3 * d, d, ws.qkv, d, nullptr, 0, nin, no_out,
                                 0, s, &qc)));
                TRY(attn_history_cached(cfg, tau_l, ws.qkv, d, scen, beh, scratch_cache, 0, ws.o, d, s));
            } else {
                qc.which0 = 1;
                TRY(rt(gemm_bf16(EPI_STORE_BF16, ws.xb, d, pw.wqkv + (size_t)d * d * 2, (int)T, 2 * d, d, ws.qkv, d,
                                 nullptr, 0, nin, no_out, 0, s, &qc)));
            }
            const RowNormIn nin_c{ws.ss + (size_t)T * np, np, 1.f / (float)d, cfg->rms_eps};
            TRY(rt(gemm_bf16(EPI_STORE_BF16, ws.xb + (size_t)T * d * 2, d, pw.wqkv, m_total, 3 * d, d, ws.qkv + crow,
                             3 * d, nullptr, 0, nin_c, no_out, 0, s)));
        } else {
            // one fused projection over both kinds of rows; keys / values of the history rows into layer 0
            // of the scratch cache through rows, attention inside the subsequences
            TRY(rt(gemm_bf16(EPI_STORE_BF16, ws.xb, d, pw.wqkv, (int)R, 3 * d, d, ws.qkv, 3 * d, nullptr, 0, nin, no_out,
                             0, s)));
            TRY(attn_history_strided(cfg, tau_l, q, k, v, 3 * d, scen, beh, scratch_cache, 0, hist_out ? ws.o : nullptr,
                                     d, s));
        }
        // candidate rows: the whole history of this layer plus themselves
        TRY(attn_sumi_strided(cfg, tau_l, scratch_cache, 0, q + crow, k + crow, v + crow, 3 * d, cand_off, m_total,
                              m_max, cand_scen, cand_beh, ws.o + (size_t)T * d * 2, d, s));
        // output projection and feed-forward on the rows that go on: all of them, or the candidates only
        const int64_t r0 = hist_out ? 0 : T, nr = R - r0;
        if (nr == 0) continue;
        const RowNormIn nin_r{ws.ss + (size_t)r0 * np, np, 1.f / (float)d, cfg->rms_eps};
        const RowNormOut nout_r{ws.ss + (size_t)r0 * np, ws.xb + (size_t)r0 * d * 2, d};
        float *x_r = ws.x32 + (size_t)r0 * d, *h_r = ws.h32 + (size_t)r0 * d;
        uint8_t *u_r = ws.u + (size_t)r0 * F * 2;  // r0 is a multiple of 64: whole groups of 16 rows
        TRY(rt(gemm_bf16(EPI_RESID_F32, ws.o + (size_t)r0 * d * 2, d, pw.wo, (int)nr, d, d, h_r, d, x_r, d, no_in,
                         nout_r, 0, s)));
        TRY(rt(gemm_bf16(EPI_GELU_BF16, ws.xb + (size_t)r0 * d * 2, d, pw.w1, (int)nr, F, d, u_r, F, nullptr, 0, nin_r,
                         no_out, kTiledC, s)));
        TRY(rt(gemm_bf16(EPI_RESID_F32, u_r, F, pw.w2, (int)nr, d, F, x_r, d, h_r, d, no_in, last ? no_out : nout_r,
                         kTiledA, s)));
    }
    if (y_hist && T) TRY(rt(hipMemcpyAsync(y_hist, ws.x32, (size_t)T * d * 4, hipMemcpyDeviceToDevice, s)));
    if (m_total)
        TRY(rt(hipMemcpyAsync(y_cand, ws.x32 + (size_t)T * d, (size_t)m_total * d * 4, hipMemcpyDeviceToDevice, s)));
    return CLIMBER_OK;
}

int climber_sumi_score(const climber_config *cfg, const climber_weights *weights, const float *tau,
                       const climber_kv_cache *cache, const void *x_cand, const int32_t *cand_off,
                       int32_t m_total, int32_t m_max, const int32_t *cand_scen,
                       const int32_t *cand_beh, float *y_cand, void *workspace, size_t ws_bytes,
                       void *stream)
{
    TRY(check_score_args(cfg, weights, tau, cache, x_cand, cand_off, m_total, m_max, cand_scen, cand_beh,
                         y_cand));
    if (!workspace) return CLIMBER_ERR_NULL;
    if ((uintptr_t)workspace % 256 != 0) return CLIMBER_ERR_ALIGN;
    Workspace ws = carve(cfg, m_total, workspace);
    if (ws_bytes < ws.total) return CLIMBER_ERR_BUFSIZE;
    return score_layers(cfg, weights, tau, cache, x_cand, cand_off, m_total, m_max, cand_scen, cand_beh,
                        y_cand, ws, (hipStream_t)stream);
}

int climber_sumi_score_static(const climber_config *cfg, const climber_weights *weights,
                              const float *tau, const climber_kv_cache *cache, const void *x_cand,
                              const int32_t *cand_off, int32_t m_total, int32_t m_max,
                              const int32_t *cand_scen, const int32_t *cand_beh, float *y_cand,
                              void *stream)
{
    TRY(check_score_args(cfg, weights, tau, cache, x_cand, cand_off, m_total, m_max, cand_scen, cand_beh,
                         y_cand));
    // the weights must come prepacked: packing them here would need room for them in the scratch array
    if (!weights->packed) return CLIMBER_ERR_NULL;
    if (carve(cfg, m_total, nullptr, false).total > CLIMBER_STATIC_SCRATCH_BYTES) return CLIMBER_ERR_BUFSIZE;
    uint8_t *base = nullptr;
    TRY(static_scratch(&base));
    Workspace ws = carve(cfg, m_total, base, false);
    return score_layers(cfg, weights, tau, cache, x_cand, cand_off, m_total, m_max, cand_scen, cand_beh,
                        y_cand, ws, (hipStream_t)stream);
}

}  // extern "C"
