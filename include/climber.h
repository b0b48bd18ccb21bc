/*
 * climber.h -- C ABI of the MI355X-native Climber serving hot path.
 *
 * The library implements the serving flow of Climber (arXiv 2502.09888, Sec. 3.2
 * "Deployment"): a user's behaviour history is encoded once, its per-layer keys
 * and values are kept in a cache in device memory, and M candidate items are then
 * scored in one batch ("single user, multiple items"): every candidate attends to
 * the whole cached history plus itself and never to another candidate.  The
 * attention is the Adaptive Transformer Layer of Sec. 3.1.3, Eq. (3): logits
 * R = qk_scale * Q K^T are divided by a temperature looked up per query row from a
 * (scenario, behaviour) table before the softmax.  History tokens only attend
 * inside their own subsequence (multi-scale sequence extraction, Sec. 3.1.2), i.e.
 * block-diagonal attention over equal subsequences of `sub_len` tokens.
 *
 * General rules
 *  - Every function returns 0 (CLIMBER_OK) or a negative CLIMBER_ERR_* code;
 *    climber_strerror() names it.  No exceptions, no output on stderr.
 *  - "dev" pointers are device (HBM) addresses owned by the caller; the library
 *    never allocates, frees or keeps them beyond what is documented for the KV
 *    cache handle.  "host" pointers are ordinary host memory, read during the call.
 *  - All device work is enqueued on the caller's stream (`stream` is a hipStream_t
 *    passed as void*; NULL is the default stream).  Compute calls do not
 *    synchronise; they return after the launches are enqueued.
 *  - Arguments are validated on the host before anything is launched; a failed
 *    call has launched nothing.  Device-resident ids cannot be checked on the
 *    host: scenario / behaviour ids outside the table are clamped into range by
 *    the kernels (results for such rows are then those of the clamped id).
 *    Temperatures must be finite and > 0; this is the caller's contract (a
 *    non-positive entry gives unspecified values for the rows that use it, never
 *    an out-of-bounds access).  climber_check_inputs() checks both on the device
 *    and reports into a caller-owned status word.
 *  - Packed batches: the histories of the B users of a batch are stored back to
 *    back with per-user padded lengths; user b owns rows
 *    tok_off[b] .. tok_off[b] + hist_len_padded[b] - 1 of every per-token array,
 *    of which the first hist_len[b] are valid.  Padded rows are never read as
 *    keys/values (they may hold anything, NaN included) and produce zeros as
 *    query rows.  Candidates are packed with device offsets cand_off[B+1].
 *  - An array of zero length may be passed as NULL: with m_total == 0 the per-candidate pointers
 *    (rows, ids, outputs) are not looked at and nothing is launched for the candidates.
 *  - Activations are token-major: q/k/v are [rows][n_heads][d_head], attention
 *    outputs and hidden states are [rows][d_model], d_model = n_heads * d_head.
 *
 * Precision paths
 *  - CLIMBER_F32 : everything fp32 (reference path; any d_head <= 256).
 *  - CLIMBER_BF16: bf16 storage, bf16 MFMA products with fp32 accumulation, fp32
 *    softmax statistics, probabilities rounded to bf16 before the P V product;
 *    requires d_head == 64, padded history lengths that are multiples of 64 and
 *    sub_len == 0 or a multiple of 128.
 *    A candidate's result does not depend on which other candidates are scored with it (the
 *    mask of Sec. 3.2); on this path it is bitwise the same however the candidates are chunked or
 *    ordered as long as its logits are of ordinary size.  With large logits the kernel picks the
 *    form of its softmax (scale folded into the query / applied in fp32 / running maximum) per
 *    wavefront or workgroup from the rows it holds, so a candidate's rounding can then differ
 *    with its neighbours in the tile; every form is within the path's tolerance.
 */
#ifndef CLIMBER_H
#define CLIMBER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CLIMBER_OK 0
#define CLIMBER_ERR_NULL (-1)        /* a required pointer is NULL */
#define CLIMBER_ERR_SHAPE (-2)       /* a size is <= 0 or inconsistent (d_model != H*d_head ...) */
#define CLIMBER_ERR_ALIGN (-3)       /* padding / multiple-of / pointer alignment rule violated */
#define CLIMBER_ERR_RANGE (-4)       /* layer index, length or offset out of range */
#define CLIMBER_ERR_TAU (-5)         /* qk_scale / rms_eps not finite or not positive */
#define CLIMBER_ERR_BUFSIZE (-6)     /* caller buffer (cache, workspace) too small */
#define CLIMBER_ERR_UNSUPPORTED (-7) /* valid request the selected precision path cannot run */
#define CLIMBER_ERR_RUNTIME (-8)     /* a HIP runtime call failed (no device, bad stream ...) */

#define CLIMBER_F32 0
#define CLIMBER_BF16 1

#define CLIMBER_HIST_CAUSAL 1 /* flags bit 0: history token i only sees j <= i of its subsequence */
/* Path selection, results equal to within rounding.  The bf16 history pass has two routes where
 * sub_len is 128 or 256: one kernel that stores the cache blocks and attends (default), or cache
 * writer + tiled attention (the route of every other sub_len). */
#define CLIMBER_HIST_TWO_KERNEL 2 /* flags bit 1: always take the cache writer + tiled attention route */
/* The stack's fused QKV projection writes history keys / values into the cache from its epilogue
 * (default), or stores them as rows that the history pass then copies into the cache. */
#define CLIMBER_QKV_VIA_ROWS 4    /* flags bit 2: keys / values go through rows */

#define CLIMBER_MODE_HISTORY 0
#define CLIMBER_MODE_CANDIDATE 1

/* Hyper-parameters.  Plain data, passed by pointer, copied where kept. */
typedef struct climber_config {
    int32_t n_layers; /* layers of the stack (>= 1); attention-only use: number of cache layers */
    int32_t d_model;  /* = n_heads * d_head */
    int32_t n_heads;
    int32_t d_head;
    int32_t d_ffn;    /* feed-forward hidden width; ignored by the attention-only calls */
    int32_t n_scen;   /* temperature table rows (scenarios) */
    int32_t n_beh;    /* temperature table columns (behaviours / extraction strategies) */
    int32_t sub_len;  /* subsequence length n_k of Sec. 3.1.2; 0 = one subsequence */
    int32_t dtype;    /* CLIMBER_F32 | CLIMBER_BF16 */
    int32_t flags;    /* CLIMBER_HIST_CAUSAL | CLIMBER_HIST_TWO_KERNEL | CLIMBER_QKV_VIA_ROWS */
    float qk_scale;   /* multiplies Q K^T before the temperature divide; Eq. (3) literally = 1 */
    float rms_eps;    /* epsilon of the RMSNorm in the layer stack */
} climber_config;

/* One layer's weights: device pointers, row-major, element type = config dtype (bf16 / fp32).
 *   g1 [d]   gain of the pre-attention RMSNorm      wqkv [d][3d]  columns Q heads | K heads | V heads
 *   wo [d][d]                                       g2 [d]   gain of the pre-FFN RMSNorm
 *   w1 [d][d_ffn]                                   w2 [d_ffn][d]
 * Layer (f_QKV and f_FFN of Eq. (3) made concrete; the paper does not fix these details):
 *   qkv = RMSNorm(x; g1) wqkv;  o = attention;  h = x + o wo;  y = h + GELU_erf(RMSNorm(h; g2) w1) w2 */
typedef struct climber_layer_weights {
    const void *g1, *wqkv, *wo, *g2, *w1, *w2;
} climber_layer_weights;

typedef struct climber_weights {
    int32_t n_layers;                    /* must equal config.n_layers */
    const climber_layer_weights *layers; /* host array of n_layers entries */
    const void *packed;                  /* dev, or NULL.  The buffer climber_pack_weights filled from
                                            these weights: climber_history_encode / climber_sumi_score
                                            then read it (and never `layers`, which may be NULL)
                                            instead of repacking the weights on every call. */
} climber_weights;

/* Opaque host-side handle describing a KV cache that lives in a caller-owned device buffer. */
typedef struct climber_kv_cache climber_kv_cache;

const char *climber_strerror(int code);

/* ---- KV cache (Sec. 3.2: "multi-layered key-value cache vectors from user features") ----------
 * The cache holds, for each of config.n_layers layers, the keys and values of every (padded)
 * history token of the batch, in a layout private to the library (for bf16: MFMA operand
 * fragments of 32-key blocks, so that the candidate pass streams it with linear 16-byte
 * accesses; padded slots are stored as zeros).  It is immutable between encodes, so any
 * number of scoring calls, on any streams, may read it concurrently.
 */

/* Bytes the device buffer of a cache must have.  hist_len_padded: host [B].  Returns 0 on any
 * invalid argument. */
size_t climber_kv_cache_bytes(const climber_config *cfg, int32_t B, const int32_t *hist_len_padded);

/* Create the handle.  hist_len, hist_len_padded: host [B], copied.  dev_buf: dev, `bytes` long,
 * 256-byte aligned, owned by the caller and must outlive the handle's use.  A small descriptor
 * (lengths, offsets, schedule) is copied into the head of dev_buf with a synchronous copy; this
 * is the only call of the library that synchronises.  0 <= hist_len[b] <= hist_len_padded[b];
 * B >= 1; sum of padded lengths < 2^31 / d_model.
 * Errors: NULL, SHAPE, ALIGN (padding rule of the dtype), RANGE, BUFSIZE, UNSUPPORTED, RUNTIME. */
int climber_kv_cache_create(const climber_config *cfg, int32_t B, const int32_t *hist_len,
                            const int32_t *hist_len_padded, void *dev_buf, size_t bytes,
                            climber_kv_cache **out);

/* Frees the host handle only; the device buffer stays with the caller.  NULL is accepted. */
int climber_kv_cache_destroy(climber_kv_cache *cache);

/* Total padded history rows of the batch (= tok_off[B]); negative error code on NULL. */
int64_t climber_kv_cache_rows(const climber_kv_cache *cache);

/* ---- attention-only entry points (caller supplies Q/K/V of one layer) ------------------------- */

/* History side of one layer (Eq. (3) restricted to a subsequence, Sec. 3.1.2):
 *  1. stores k, v of all history tokens into cache layer `layer`;
 *  2. if o_hist != NULL, block-diagonal attention of the history tokens:
 *       o_i = sum_j softmax_j( qk_scale <q_i,k_j> / tau[scen_i][beh_i] ) v_j
 *     over the valid tokens j of i's subsequence (j <= i as well under CLIMBER_HIST_CAUSAL).
 * tau_layer: dev [n_scen][n_beh] fp32.  q (may be NULL iff o_hist is NULL), k, v: dev
 * [rows][H][d_head] of the config dtype, rows = climber_kv_cache_rows().  scen, beh: dev int32
 * [rows] (only read when o_hist != NULL).  o_hist: dev [rows][d_model] of the config dtype;
 * padded rows receive zeros. */
int climber_attn_history(const climber_config *cfg, const float *tau_layer, const void *q,
                         const void *k, const void *v, const int32_t *scen, const int32_t *beh,
                         climber_kv_cache *cache, int32_t layer, void *o_hist, void *stream);

/* SUMI attention of one layer (mask of Sec. 3.2, temperature of Eq. (3)): for candidate c of
 * user b
 *     o_c = softmax over { all hist_len[b] cached history keys of b, c's own key } of
 *           qk_scale <q_c, k> / tau[cscen_c][cbeh_c],   applied to the matching values.
 * q_c, k_c, v_c: dev [m_total][H][d_head]; cand_off: dev int32 [B+1], cand_off[0] = 0,
 * non-decreasing, cand_off[B] = m_total; m_max: host value, must be >= max_b (cand_off[b+1] -
 * cand_off[b]): it sizes the launch, and m_max * B == m_total tells the library that every user
 * has exactly m_max candidates.  A smaller m_max breaks the contract (rows may then be left
 * unwritten or scored against the wrong user's history, never an out-of-bounds access);
 * climber_check_inputs reports it.
 * cand_scen, cand_beh: dev int32 [m_total].  o_c: dev [m_total][d_model].
 * Scoring a candidate set in chunks = calling this repeatedly on the same (const) cache. */
int climber_attn_sumi(const climber_config *cfg, const float *tau_layer,
                      const climber_kv_cache *cache, int32_t layer, const void *q_c,
                      const void *k_c, const void *v_c, const int32_t *cand_off, int32_t m_total,
                      int32_t m_max, const int32_t *cand_scen, const int32_t *cand_beh, void *o_c,
                      void *stream);

/* ---- relative attention bias (Eq. (3): R = Q K^T + f_b, divided by the temperature) -----------
 * Sec. 3.1.3 names what the bias depends on (relative position and relative time, per extraction
 * strategy and scenario) and not its form.  The form of this library:
 *     bias(i, j; h) = pos_table[scen_i][beh_i][h][bp(pos_i - pos_j)]
 *                   + time_table[scen_i][beh_i][h][bt(ts_i - ts_j)]
 *     bp(d) = clip(d, -(n_pos-1)/2, (n_pos-1)/2) + (n_pos-1)/2          (n_pos odd, >= 1)
 *     bt(d) = min( floor(log2(max(|d|, 1))), n_time - 1 )               (n_time >= 1)
 * i = query row (its scenario / behaviour ids select the table row, as they select its temperature),
 * j = key; pos / ts are caller-defined integers per history row and per candidate (e.g. index in the
 * history and seconds); a candidate's own key has distance 0 in both.  The bias is added to
 * qk_scale <q_i, k_j> and the sum is divided by the row's temperature.
 * All pointers dev; tables fp32 (both precision paths); hist_pos / hist_ts: int32 [rows], 16-byte
 * aligned, padded rows may hold anything; cand_pos / cand_ts: int32 [m_total]. */
typedef struct climber_rel_bias {
    const float *pos_table;  /* [n_scen][n_beh][n_heads][n_pos] */
    const float *time_table; /* [n_scen][n_beh][n_heads][n_time] */
    int32_t n_pos, n_time;
    const int32_t *hist_pos, *hist_ts;
    const int32_t *cand_pos, *cand_ts; /* only read by climber_attn_sumi_bias */
} climber_rel_bias;

/* climber_attn_history / climber_attn_sumi with the bias term (bias != NULL; everything else as
 * documented there).  The bf16 history pass takes the cache writer + tiled attention route.
 * Additional errors: CLIMBER_ERR_NULL (bias or a pointer it needs), _SHAPE (n_pos even or < 1,
 * n_time < 1), _ALIGN (hist_pos / hist_ts). */
int climber_attn_history_bias(const climber_config *cfg, const float *tau_layer, const void *q,
                              const void *k, const void *v, const int32_t *scen, const int32_t *beh,
                              climber_kv_cache *cache, int32_t layer, void *o_hist,
                              const climber_rel_bias *bias, void *stream);
int climber_attn_sumi_bias(const climber_config *cfg, const float *tau_layer,
                           const climber_kv_cache *cache, int32_t layer, const void *q_c,
                           const void *k_c, const void *v_c, const int32_t *cand_off,
                           int32_t m_total, int32_t m_max, const int32_t *cand_scen,
                           const int32_t *cand_beh, void *o_c, const climber_rel_bias *bias,
                           void *stream);

/* ---- debug check of device-resident inputs -----------------------------------------------------
 * Eq. (3) divides a row's logits by tau[scen][beh]: the ids must lie inside the table and the entry
 * must be finite and > 0.  Ids, offsets and the table live in device memory, so the compute calls
 * cannot validate them on the host (they clamp ids and leave the rest to the caller's contract).
 * This call launches one small kernel on `stream` that reads, inside the given bounds only,
 *   - history rows (cache != NULL): scen / beh of the valid rows of every user of the cache
 *     (padding rows may hold anything); cand_off, B_cand, m_max are ignored;
 *   - candidate rows (cache == NULL): scen / beh [m_total], and, if cand_off != NULL, cand_off
 *     [B_cand + 1] against the rules of climber_attn_sumi (starts at 0, non-decreasing, ends at
 *     m_total, every count <= m_max);
 *   - the entries of tau_layer that the checked rows select;
 * and ORs CLIMBER_BAD_* bits into *status (dev int32; the caller zeroes it before, and reads it after
 * synchronising the stream: 0 = nothing found).  The kernel always runs to completion.
 * Errors: CLIMBER_ERR_NULL, _SHAPE (m_total < 0, B_cand < 1 with cand_off), _RUNTIME. */
#define CLIMBER_BAD_SCEN 1    /* a scenario id outside [0, n_scen) */
#define CLIMBER_BAD_BEH 2     /* a behaviour id outside [0, n_beh) */
#define CLIMBER_BAD_TAU 4     /* a selected temperature is not finite or not > 0 */
#define CLIMBER_BAD_OFFSETS 8 /* cand_off not 0-based, decreasing somewhere, or not ending at m_total */
#define CLIMBER_BAD_M_MAX 16  /* a user has more candidates than m_max */
int climber_check_inputs(const climber_config *cfg, const float *tau_layer, const int32_t *scen,
                         const int32_t *beh, const climber_kv_cache *cache, int32_t m_total,
                         const int32_t *cand_off, int32_t B_cand, int32_t m_max, int32_t *status,
                         void *stream);

/* ---- layer stack (CLIMBER_BF16 only) ---------------------------------------------------------- */

/* Bytes of scratch the stack calls need for up to max_rows rows (history rows or candidates). */
size_t climber_workspace_bytes(const climber_config *cfg, int64_t max_rows);

/* One layer of the stack on the history rows (mode HISTORY: writes cache layer `layer`, attends
 * block-diagonally) or on candidate rows (mode CANDIDATE: SUMI attention against cache layer
 * `layer`).  x_in, x_out: dev fp32 [rows][d_model] residual stream (x_out may be NULL in HISTORY
 * mode: then only the layer's K/V are produced, which is all the last layer of an encode needs;
 * x_out may alias x_in).  ids: per-row scenario / behaviour ids of the rows being processed.
 * cand_off / m_total / m_max as in climber_attn_sumi (ignored in HISTORY mode).
 * workspace: dev, >= climber_workspace_bytes(cfg, rows), 256-byte aligned. */
int climber_layer_forward(const climber_config *cfg, const climber_layer_weights *w,
                          const float *tau_layer, int32_t layer, int32_t mode,
                          climber_kv_cache *cache, const float *x_in, float *x_out,
                          const int32_t *scen, const int32_t *beh, const int32_t *cand_off,
                          int32_t m_total, int32_t m_max, void *workspace, size_t ws_bytes,
                          void *stream);

/* The projections read their weights as MFMA operand fragments with the RMSNorm gains multiplied
 * in (f_QKV / f_FFN of Eq. (3)); the stack calls bring `layers` into that form in their workspace
 * on every call (~1 % of a step).  A caller whose weights do not change can do it once:
 * climber_pack_weights fills `packed` (dev, 256-byte aligned, >= climber_packed_weights_bytes(cfg),
 * 0 on an invalid config) from weights->layers on `stream`; the caller then sets weights->packed
 * to that buffer, which must stay unchanged while calls that were given it are running.  Results
 * are bitwise the same either way.  Errors: CLIMBER_ERR_NULL, _SHAPE (n_layers), _ALIGN,
 * _BUFSIZE, _UNSUPPORTED (not the bf16 stack), _RUNTIME. */
size_t climber_packed_weights_bytes(const climber_config *cfg);
int climber_pack_weights(const climber_config *cfg, const climber_weights *weights, void *packed,
                         size_t bytes, void *stream);

/* History encode (first phase of the serving flow, Sec. 3.2): runs the packed history embeddings
 * x_hist (dev bf16 [rows][d_model]) through all layers and fills every layer of the cache.  The
 * last layer stops after its K/V are stored.  tau: dev fp32 [n_layers][n_scen][n_beh].
 * workspace must hold climber_workspace_bytes(cfg, rows). */
int climber_history_encode(const climber_config *cfg, const climber_weights *weights,
                           const float *tau, const void *x_hist, const int32_t *scen,
                           const int32_t *beh, climber_kv_cache *cache, void *workspace,
                           size_t ws_bytes, void *stream);

/* Candidate scoring (second phase): x_cand dev bf16 [m_total][d_model] -> y_cand dev fp32
 * [m_total][d_model], the candidates' final-layer hidden states (the paper's scalar score needs
 * its fusion module and an unspecified head on top of these).  workspace must hold
 * climber_workspace_bytes(cfg, m_total). */
int climber_sumi_score(const climber_config *cfg, const climber_weights *weights, const float *tau,
                       const climber_kv_cache *cache, const void *x_cand, const int32_t *cand_off,
                       int32_t m_total, int32_t m_max, const int32_t *cand_scen,
                       const int32_t *cand_beh, float *y_cand, void *workspace, size_t ws_bytes,
                       void *stream);

/* Training-side form of the "single user, multiple items" pattern (Sec. 3.2): the histories and the
 * candidates of a batch run through all layers TOGETHER as one packed set of rows under the mask of
 * that section (history rows: own subsequence; a candidate: its user's whole history and itself,
 * never another candidate) and nothing is cached across calls -- the forward pass behind the
 * paper's training-throughput figure.  Same result as climber_history_encode followed by
 * climber_sumi_score (bitwise for y_cand under the default flags); the output projection and
 * feed-forward launches of a layer cover both kinds of rows, and the history keys / values of the
 * layer being computed live in layer 0 of `scratch_cache` (a cache handle
 * created for this batch's histories with any number of layers; its layer 0 is overwritten).
 * y_hist: dev fp32 [rows][d_model] or NULL (then the last layer skips the history rows' attention
 * and feed-forward); y_cand: dev fp32 [m_total][d_model].  workspace must hold
 * climber_workspace_bytes(cfg, rows + m_total).  Candidate counts may differ per user (cand_off).
 * Errors as climber_history_encode / climber_sumi_score. */
int climber_sumi_forward(const climber_config *cfg, const climber_weights *weights, const float *tau,
                         const void *x_hist, const int32_t *scen, const int32_t *beh,
                         const void *x_cand, const int32_t *cand_off, int32_t m_total, int32_t m_max,
                         const int32_t *cand_scen, const int32_t *cand_beh,
                         climber_kv_cache *scratch_cache, float *y_hist, float *y_cand,
                         void *workspace, size_t ws_bytes, void *stream);

/* ---- bit-wise gating fusion (Sec. 3.1.4, Eq. (4)) and score ------------------------------------
 * The paper runs one Transformer block per subsequence ("corresponding block", Sec. 3.1.2); block k
 * turns a candidate into an output vector E(S_k), and the fusion module turns the N_b vectors of a
 * candidate into its score:
 *     G = ATL(E)                     one attention layer over the N_b rows of the candidate, every row
 *                                    seeing every row, no relative attention bias, temperature from the
 *                                    candidate's scenario only (tau_scen[scen])
 *     Y = G (.) sigmoid(f_gate(G))   f_gate: squeeze-and-excitation with equal input / output size
 *     score = head(Y)
 * As fixed by this library where the paper is silent: the fusion ATL is a layer of the stack's
 * composition (see climber_layer_weights) with weights of its own; f_gate maps the N_b * d_model
 * values of G, flattened row by row, down to d_gate, applies ReLU, and maps back (no bias vectors);
 * the head is <w_head, vec(Y)> + b_head.  Block k's E(S_k) is produced with the calls above: a
 * cache over subsequence k only (sub_len = 0), block k's weights, climber_history_encode, then
 * climber_sumi_score or climber_sumi_forward: its y_cand rows are E(S_k).
 * e: dev fp32 [m_total][n_blocks][d_model]; cand_scen: dev int32 [m_total]; y: dev fp32 like e, or
 * NULL; score: dev fp32 [m_total].  CLIMBER_BF16, d_head = 64, 1 <= n_blocks <= 16, d_gate a
 * multiple of 128 and <= n_blocks * d_model.  e, y, w_down, w_up, w_head: 16-byte aligned.
 * workspace: climber_bgf_workspace_bytes(), 256-byte aligned.  Errors: CLIMBER_ERR_NULL, _SHAPE, _UNSUPPORTED, _ALIGN, _RANGE, _BUFSIZE, _RUNTIME. */
typedef struct climber_bgf_weights {
    climber_layer_weights atl; /* fusion layer, bf16, shapes of a stack layer */
    const void *w_down;        /* dev bf16 [n_blocks * d_model][d_gate] */
    const void *w_up;          /* dev bf16 [d_gate][n_blocks * d_model] */
    const float *w_head;       /* dev fp32 [n_blocks * d_model] */
    const float *tau_scen;     /* dev fp32 [n_scen] */
    float b_head;
    int32_t n_blocks, d_gate;
} climber_bgf_weights;
size_t climber_bgf_workspace_bytes(const climber_config *cfg, int32_t n_blocks, int32_t d_gate,
                                   int64_t m_total);
int climber_bgf_score(const climber_config *cfg, const climber_bgf_weights *w, const float *e,
                      const int32_t *cand_scen, int32_t m_total, float *y, float *score,
                      void *workspace, size_t ws_bytes, void *stream);

/* climber_sumi_score for callers that cannot allocate or hand over device memory for scratch: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same kernels and bitwise the same y_cand as climber_sumi_score, but the scratch lives in a fixed
 * array of CLIMBER_STATIC_SCRATCH_BYTES inside the library (one per GPU, held until the process
 * ends) instead of a caller's workspace, and the call allocates and frees nothing.
 *  - weights->packed must be set (climber_pack_weights): CLIMBER_ERR_NULL otherwise.
 *  - m_total is limited by the array: climber_workspace_bytes(cfg, m_total) minus
 *    climber_packed_weights_bytes(cfg) must not exceed CLIMBER_STATIC_SCRATCH_BYTES
 *    (2512 candidates at d_model 512, d_ffn 2048); beyond that CLIMBER_ERR_BUFSIZE and nothing is
 *    launched.
 *  - All calls on one GPU share that GPU's array: calls that may overlap on one GPU (different
 *    streams, different threads) race; serialise them.  The first call on a GPU looks the array's
 *    address up (no allocation); make that call outside a graph capture.
 * Other errors as climber_sumi_score. */
#define CLIMBER_STATIC_SCRATCH_BYTES (32u << 20)
int climber_sumi_score_static(const climber_config *cfg, const climber_weights *weights,
                              const float *tau, const climber_kv_cache *cache, const void *x_cand,
                              const int32_t *cand_off, int32_t m_total, int32_t m_max,
                              const int32_t *cand_scen, const int32_t *cand_beh, float *y_cand,
                              void *stream);

#ifdef __cplusplus
}
#endif
#endif /* CLIMBER_H */
