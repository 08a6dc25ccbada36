/*
 * ssd.h -- C ABI of the MI355X (gfx950) self-speculative decoding library.
 *
 * The library runs the batch-1 decoder forward that ConfLayers accelerates: a draft forward
 * with a layer skip set, the full-model verification of the drafted tokens, greedy
 * acceptance, and the per-layer entropy confidence that ranks layers for skipping, plus the
 * host-side skip-set selection and periodic search that consume those confidences.
 *
 * Conventions
 *   - Every function returns SSD_OK (0) or a negative error code; nothing throws.
 *   - "device" pointers are HIP device memory owned by the caller (e.g. torch tensors) and
 *     only borrowed; "host" pointers are ordinary host memory.  The library owns nothing on
 *     the device: KV cache, activations and scratch live in the caller's workspace buffer.
 *   - All device work is enqueued on the stream given to ssd_create.  Calls that return
 *     values through host pointers synchronise that stream before returning.
 *   - Matrices are row-major [out_features][in_features], fp32, bf16 or fp16.
 *   - Decoding state: committed tokens t_0..t_{n-1}; the cache holds verified K/V for
 *     positions 0..n-2; the last committed token is "pending" (not yet in the cache).
 *   - Call order: create -> set_workspace + load_weights -> prefill ->
 *       { decode | draft_step -> verify -> accept }*      anything else is SSD_ESTATE.
 *   - Arguments are validated on the host before anything is launched; an error return
 *     means no device work was enqueued by that call (SSD_EHIP excepted).
 *   - A context is not thread-safe; use one context per stream.
 */
#ifndef SSD_H
#define SSD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The shared library is built with hidden visibility: exactly the functions declared here are exported. */
#define SSD_API __attribute__((visibility("default")))

enum {
    SSD_OK = 0,
    SSD_EINVAL = -1,    /* bad argument */
    SSD_ESTATE = -2,    /* call order violated */
    SSD_ECAPACITY = -3, /* max_seq / max_k / row limits exceeded */
    SSD_ENOMEM = -4,    /* workspace missing or too small */
    SSD_EHIP = -5       /* HIP runtime error; text via ssd_last_error */
};

#define SSD_MAX_K 15        /* largest draft length: k + 1 rows fill one 16-column MFMA tile */
#define SSD_MAX_LAYERS 128  /* deepest model a context accepts (fixed-size per-layer result slots in the workspace) */
#define SSD_MAX_WINDOW 4096 /* largest context window of the confidence extraction (positions kept on the device) */
#define SSD_PREFILL_ROWS 512 /* most prompt rows processed per pass of the weights (64 or 16 where a shape does not fit
                                the 128 x 128 or the 64-row tiling: widths not multiples of 128, fp32 weights) */

typedef struct ssd_ctx ssd_ctx;

/* Decoder shape and numeric options.  d_model = n_heads * head_dim is not required, but
 * head_dim must be 64 or 128, n_heads a multiple of n_kv_heads, n_layers at most SSD_MAX_LAYERS, and d_model,
 * d_ffn, n_heads*head_dim, n_kv_heads*head_dim and vocab multiples of 16. */
typedef struct {
    int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab, max_seq;
    float rms_eps, rope_base;
    int32_t weight_dtype; /* 0 = fp32, 1 = bf16, 2 = fp16 (the precision of Section 4.1.1): element type of the
                             weight matrices */
    int32_t conf_taps;    /* 2: confidence of a layer = mean over its post-attention and post-MLP hidden
                             states (Section 3.1: "FFNN and Attention" hidden states); 1: post-MLP only */
    float conf_clamp;     /* logits are clamped to [-conf_clamp, conf_clamp] before Eq. 1 */
    float conf_eps;       /* epsilon of Eq. 2 */
    int32_t max_k;        /* largest k that draft_step / verify will be called with (1..SSD_MAX_K) */
    int32_t kv_dtype;     /* 0 = fp32, 1 = bf16, 2 = fp16: element type of the KV cache (K after the rotary embedding and V
                             are rounded to it, nearest-even, when stored); independent of weight_dtype */
    int32_t conf_window;  /* context window of the confidence extraction (100 tokens, Section 4.1.1): the workspace keeps the
                             hidden-state taps of the last conf_window processed positions for ssd_window_confidence;
                             0 = none kept (0..SSD_MAX_WINDOW) */
} ssd_config;

/* Device pointers to the weights.  The per-layer members are HOST arrays of n_layers DEVICE
 * pointers.  Norm gains are fp32 [d_model]; every matrix has weight_dtype elements:
 * embed, lm_head [vocab][d_model]; wq [n_heads*head_dim][d_model]; wk, wv
 * [n_kv_heads*head_dim][d_model]; wo [d_model][n_heads*head_dim]; wg, wu [d_ffn][d_model];
 * wd [d_model][d_ffn]. */
typedef struct {
    const void *embed, *lm_head;
    const float *final_norm;
    const float *const *attn_norm;
    const void *const *wq, *const *wk, *const *wv, *const *wo;
    const float *const *mlp_norm;
    const void *const *wg, *const *wu, *const *wd;
} ssd_weights;

typedef struct {
    int64_t cycles, drafted, accepted, committed; /* alpha = accepted / drafted, M = accepted / cycles (Section 4.1.2) */
    int64_t decode_steps, draft_steps, verify_rows, confidence_rows;
    int32_t n_tokens;                              /* committed tokens n (prompt included) */
    int32_t state;
} ssd_stats;

/* ---- lifetime ------------------------------------------------------------------------- */

/* Validates cfg and creates a host-side context bound to hip_stream (a hipStream_t, may be
 * NULL for the default stream).  No device memory is touched. */
SSD_API int ssd_create(const ssd_config *cfg, void *hip_stream, ssd_ctx **out);

/* Bytes of device workspace a context with this cfg needs (KV cache for max_seq positions,
 * rotary table, activations for max(max_k + 1, SSD_PREFILL_ROWS) rows, hidden-state taps,
 * logits, split-attention partials).  0 if cfg is invalid. */
SSD_API size_t ssd_workspace_bytes(const ssd_config *cfg);

/* Hands the context its workspace: device memory, 256-byte aligned, at least
 * ssd_workspace_bytes(cfg) long, borrowed until ssd_destroy.  Uploads the rotary table.
 * SSD_ENOMEM if dev is NULL or bytes too small. */
SSD_API int ssd_set_workspace(ssd_ctx *ctx, void *dev, size_t bytes);

/* Section 3 / Figure 2: the same weights serve the draft and the target model.  Borrows the
 * device pointers (no copy, no repack); the caller keeps the tensors alive. */
SSD_API int ssd_load_weights(ssd_ctx *ctx, const ssd_weights *w);

/* Forget the sequence (back to the state after load_weights); weights and workspace stay. */
SSD_API int ssd_reset(ssd_ctx *ctx);
SSD_API void ssd_destroy(ssd_ctx *ctx);
SSD_API const char *ssd_last_error(const ssd_ctx *ctx);
SSD_API int ssd_get_stats(const ssd_ctx *ctx, ssd_stats *out);

/* ---- generation step (Figure 2, "generation") ----------------------------------------- */

/* Full-model forward over the n prompt tokens (host int32), at most SSD_PREFILL_ROWS rows per pass.
 * Fills the cache for positions 0..n-1, keeps the hidden-state taps of the last row, and
 * commits the greedy first new token (returned in *first_token_out, host). n + 1 tokens are
 * then committed.  SSD_ECAPACITY if n + 1 > max_seq. */
SSD_API int ssd_prefill(ssd_ctx *ctx, const int32_t *tokens, int n, int32_t *first_token_out);

/* One vanilla autoregressive step with the full model (the baseline of Section 4.1.1):
 * feeds the pending token, commits and returns the greedy next token. */
SSD_API int ssd_decode(ssd_ctx *ctx, int32_t *token_out);

/* Draft model of Section 3: the target model without the layers in the skip set S
 * (skip_mask[l] != 0 means layer l is in S; a skipped layer leaves the residual stream
 * unchanged, reads and writes no cache).  Generates k greedy tokens one after another,
 * starting from the pending token; executed layers write draft K/V at positions n-1..n+k-2.
 * draft_out: host [k]; draft_maxprob_out: host [k] or NULL (softmax max-probability of each
 * drafted token).  SSD_ECAPACITY if n + k > max_seq or k > max_k. */
SSD_API int ssd_draft_step(ssd_ctx *ctx, const uint8_t *skip_mask, int k, int32_t *draft_out,
                   float *draft_maxprob_out);

/* The same with the attention and the MLP sub-block of every layer skipped separately -- the two modules whose hidden
 * states Section 3.1 scores one by one (the layer-skipping baselines of Section 2 skip at this granularity):
 * sub_mask is host [2 * n_layers], sub_mask[2l] != 0 leaves out the attention sub-block of layer l (no projections, no
 * cache write at the draft positions), sub_mask[2l+1] != 0 its MLP sub-block.  ssd_draft_step(skip_mask) equals this
 * call with both entries of every skipped layer set.  Verification is unchanged. */
SSD_API int ssd_draft_step_sub(ssd_ctx *ctx, const uint8_t *sub_mask, int k, int32_t *draft_out,
                               float *draft_maxprob_out);

/* Confidence-aware drafting (Section 3: once a skip set is found the candidate tokens are
 * generated with the confidence-aware draft exit of the layer-skipping baseline the paper builds
 * on; the paper gives no threshold, gamma is the caller's).  Same draft model and cache effects as
 * ssd_draft_step, but tokens are drafted one at a time and drafting stops after the first token
 * whose draft softmax max-probability is below gamma (that token is kept), or after k_max tokens.
 * draft_out: host [k_max]; draft_maxprob_out: host [k_max] or NULL; *k_out (host) receives the
 * number of tokens drafted (1..k_max), which is the k to pass to ssd_verify / ssd_accept.
 * The comparison p < gamma is taken in fp32 on the max-probability the device computed.
 * SSD_ECAPACITY if n + k_max > max_seq or k_max > max_k; SSD_EINVAL if gamma is NaN. */
SSD_API int ssd_draft_adaptive(ssd_ctx *ctx, const uint8_t *skip_mask, int k_max, float gamma,
                       int32_t *draft_out, float *draft_maxprob_out, int32_t *k_out);

/* Verification (Section 1: drafted tokens "verified by the target model in a single forward
 * pass"): the full model over the rows [pending, draft_1..draft_k] at positions n-1..n-1+k,
 * causal inside the block; overwrites the K/V of every layer at those positions and captures
 * the hidden-state taps of all k+1 rows.  target_out: host [k+1], the greedy token after
 * each row.  Must follow ssd_draft_step / ssd_draft_adaptive with the same k; the draft tokens passed here are
 * the ones verified. */
SSD_API int ssd_verify(ssd_ctx *ctx, const int32_t *draft, int k, int32_t *target_out);

/* Greedy acceptance: a = largest m with draft_j == target_{j-1} for all 1 <= j <= m; commits
 * draft_1..draft_a and target_a (a + 1 tokens), which becomes the pending token; cache
 * entries beyond position n-1+a are stale and never read again. Host in, host out; the device-side
 * state update is enqueued on the stream, the call does not synchronise. */
SSD_API int ssd_accept(ssd_ctx *ctx, const int32_t *draft, const int32_t *target, int k,
               int32_t *n_accepted_out, int32_t *next_token_out);

/* Test hook: after ssd_verify, commit n_accepted drafted tokens and next_token regardless of
 * what the device computed (re-synchronises with an external reference after a sub-tolerance
 * arg-max tie).  draft: host [k] as passed to ssd_verify. */
SSD_API int ssd_force_commit(ssd_ctx *ctx, const int32_t *draft, int k, int n_accepted, int32_t next_token);

/* Copies fp32 logits rows [row_begin, row_begin + n_rows) of the last prefill (1 row),
 * decode (1 row), draft_step (k rows, one per drafted token) or verify (k+1 rows) to host
 * memory [n_rows][vocab]. */
SSD_API int ssd_copy_logits(ssd_ctx *ctx, int row_begin, int n_rows, float *logits_out);

/* ---- layer optimisation search step (Section 3.1) -------------------------------------- */

/* Per-layer confidence (Eq. 1-4) of rows [row_begin, row_begin+n_rows) of the last verify
 * (rows 0..k) or prefill (row 0): every tapped hidden state goes through the final RMSNorm
 * and the shared LM head; the fp32 logits are clamped, soft-maxed (Eq. 1), and
 * confidence = 1 - H / log(vocab) with H = -sum p log(p + eps) (Eq. 2-4).
 *   conf_out       host [n_rows][n_layers]: mean over the layer's taps (conf_taps of them)
 *   tap_conf_out   host [n_rows][n_layers][2] or NULL: post-attention, post-MLP confidence
 *   tap_maxprob_out, tap_argmax_out  host [n_rows][n_layers][2] or NULL */
SSD_API int ssd_layer_confidence(ssd_ctx *ctx, int row_begin, int n_rows, float *conf_out,
                         float *tap_conf_out, float *tap_maxprob_out, int32_t *tap_argmax_out);

/* Confidence over the context window (Section 4.1.1, "context window" of 100 tokens; Appendix D): Eq. 1-4 on every
 * tapped hidden state of each of the last conf_window positions that the full model processed with a committed input
 * token -- the last prompt position, then rows 0..a of every verification (ssd_accept / ssd_force_commit put them into
 * a ring in the workspace; vanilla ssd_decode steps capture no taps and leave the window as it is) -- averaged over
 * those positions.  All window rows go through the LM head in 64-row MFMA passes and one reduction; one read-back.
 *   conf_out      host [n_layers]: mean over the window of the layer's confidence (mean of its conf_taps taps)
 *   tap_conf_out  host [n_layers][2] or NULL: window means of the post-attention and post-MLP confidence
 *   n_positions_out  host or NULL: positions in the window (<= conf_window)
 * SSD_ESTATE if conf_window is 0, no sequence is prefilled or a draft is in flight. */
SSD_API int ssd_window_confidence(ssd_ctx *ctx, float *conf_out, float *tap_conf_out, int32_t *n_positions_out);

/* For callers that cannot allocate device memory while they run (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the same computation and results as ssd_layer_confidence, but every device
 * buffer the pass needs beyond the context's taps and weights -- the normalised rows, their logits, the per-row
 * results -- lives in a fixed array inside the library image (SSD_STATIC_SCRATCH_BYTES per GPU, held until the process
 * ends) instead of the workspace, 64 tap rows at a time.  Calls nothing that allocates.  SSD_ECAPACITY if 64 rows of
 * this model exceed the array (64 * (4 * vocab + 8 * d_model) bytes, e.g. a 128 256-entry vocabulary); SSD_EINVAL if
 * the context's device is not the current one.  All calls on one GPU share that GPU's array: calls that overlap in
 * time on one GPU (two contexts, two streams) race; the array keeps the last call's contents. */
#define SSD_STATIC_SCRATCH_BYTES (12u << 20)
SSD_API int ssd_layer_confidence_static(ssd_ctx *ctx, int row_begin, int n_rows, float *conf_out,
                                        float *tap_conf_out, float *tap_maxprob_out, int32_t *tap_argmax_out);

/* Eq. 5-10 parameters.  Defaults (ssd_select_defaults): lambda 0.3, w_base 2, kappa 1,
 * flat_tol 1e-3, min_ratio 0.40, max_ratio 0.60, protect_ends 1, eps 1e-8, fixed_w_max -1. */
typedef struct {
    double lambda;      /* Eq. 10 threshold sensitivity, 0.25 < lambda < 0.5 (Section 4.1.1) */
    double w_base;      /* Eq. 7 */
    double kappa;       /* w_max = kappa * (leading candidate layers with equal confidence) (Section 3.2) */
    double flat_tol;    /* two confidences are "the same value" if they differ by at most this */
    double min_ratio;   /* minimum skip ratio (Section 4.1.1) */
    double max_ratio;   /* upper end of the useful range (Section 3.2) */
    int32_t protect_ends; /* first and last layer are never candidates (Appendix B) */
    double eps;         /* epsilon of Eq. 5 and of the min-max rescale of Eq. 6 */
    double fixed_w_max; /* >= 0: use this w_max instead (0 = constant window, Section 4.3.2) */
} ssd_select_params;

SSD_API void ssd_select_defaults(ssd_select_params *p);

/* Section 3.2: standardise the confidences (Eq. 5), second-order discrete gradient rescaled
 * to [0,1] (Eq. 6), per-layer window w_i (Eq. 7), local mean / std excluding the layer
 * (Eq. 8-9), skip iff c_hat_i < mu_local - lambda * sigma_local (Eq. 10), then the skip-ratio
 * bounds.  Pure host code in double precision.  conf: host [n_layers]; mask_out: host
 * [n_layers], 1 = skip, implicitly sorted by index; n_skipped_out may be NULL;
 * margin_out: host [n_layers] or NULL, c_hat_i - (mu_local - lambda sigma_local), 0 for
 * non-candidates. */
SSD_API int ssd_select_skip(const double *conf, int n_layers, const ssd_select_params *p,
                    uint8_t *mask_out, int32_t *n_skipped_out, double *margin_out);

/* Initial draft model: uniform layer skipping (Section 3), every second candidate layer. */
SSD_API int ssd_uniform_skip(int n_layers, const ssd_select_params *p, uint8_t *mask_out);

/* ---- search check (Section 3.3) --------------------------------------------------------- */

typedef struct ssd_search ssd_search;
typedef struct {
    int32_t opt_interval; /* cycles a skip set is used before it is scored (30, Section 4.1.1) */
    double score_goal;    /* halt when mean accepted tokens per cycle reaches this (4) */
    int32_t max_rounds;   /* halt after this many scored sets */
    int32_t window;       /* confidence vectors of the last `window` cycles are averaged (100) */
} ssd_search_params;

SSD_API void ssd_search_defaults(ssd_search_params *p);
SSD_API int ssd_search_create(int n_layers, const ssd_search_params *sp, const ssd_select_params *sel,
                      ssd_search **out);
SSD_API void ssd_search_destroy(ssd_search *s);
/* Current skip set (host [n_layers]); starts as the uniform set. */
SSD_API int ssd_search_mask(const ssd_search *s, uint8_t *mask_out);
/* Feed one finished cycle: its accepted count and (optionally, may be NULL) its per-layer
 * confidences, host [n_layers] doubles.  Every opt_interval cycles the set is scored by its
 * mean accepted tokens, the best set is kept, and either the search halts (goal reached or
 * max_rounds) and the best set is adopted for good, or a new set is selected from the
 * averaged confidences.  mask_out receives the set for the next cycle; *active_out is 0
 * once the search has halted. */
SSD_API int ssd_search_observe(ssd_search *s, int n_accepted, const double *conf, uint8_t *mask_out,
                       int32_t *active_out);
/* rounds scored so far, best score so far (either may be NULL) */
SSD_API int ssd_search_status(const ssd_search *s, int32_t *rounds_out, double *best_score_out);

/* ---- measurement helpers ----------------------------------------------------------------- */

/* Streams `bytes` of device memory once through a read-only kernel `iters` times and
 * returns the mean time per pass in milliseconds (the practical HBM read ceiling of the
 * box).  dev: device pointer, 16-byte aligned; stream as in ssd_create. */
SSD_API int ssd_hbm_read_probe(const void *dev, size_t bytes, int iters, void *hip_stream, float *ms_out);

/* Per-kernel timing for roofline measurements: while a kernel id is selected, every launch of
 * that kernel is bracketed by HIP events on the context's stream (this perturbs the stream, so
 * use a separate timed pass for throughput).  ssd_profile_select resets the counters;
 * kernel_id -1 switches timing off.  ssd_profile_read synchronises the stream and returns the
 * number of bracketed launches and their summed duration in milliseconds. */
enum {
    SSD_K_GEMV_QKV = 0,    /* draft: RMSNorm + QKV GEMV + rotary + cache write */
    SSD_K_ATTENTION = 1,   /* split attention over the cache incl. the combine kernel */
    SSD_K_GEMV_O = 2,      /* draft: output projection + residual */
    SSD_K_GEMV_GATEUP = 3, /* draft: RMSNorm + gate/up GEMV + SwiGLU */
    SSD_K_GEMV_DOWN = 4,   /* draft: down projection + residual */
    SSD_K_GEMV_LMHEAD = 5, /* draft: final norm + LM head GEMV */
    SSD_K_VOCAB = 6,       /* vocabulary reduction */
    SSD_K_ROWS_QKV = 7,    /* verify: QKV MFMA GEMM */
    SSD_K_ROWS_O = 8,
    SSD_K_ROWS_GATEUP = 9,
    SSD_K_ROWS_DOWN = 10,
    SSD_K_ROWS_LMHEAD = 11, /* verify / confidence: LM head MFMA GEMM */
    SSD_K_COUNT = 12
};
SSD_API int ssd_profile_select(ssd_ctx *ctx, int kernel_id);
/* Launch mode: 1 (default) replays decode / draft / verify launch sequences as HIP graphs once a
 * sequence has been seen twice (needs a non-default stream); 0 launches kernel by kernel.  Both
 * modes run the same kernels with the same arguments and give bit-identical results. */
SSD_API int ssd_set_graphs(ssd_ctx *ctx, int enable);
SSD_API int ssd_profile_read(ssd_ctx *ctx, int64_t *launches_out, double *total_ms_out);

/* Test hook: overwrite every cache entry at positions >= the number of valid positions
 * (n - 1) with NaN, to prove stale entries are never read. */
SSD_API int ssd_kv_poison_stale(ssd_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* SSD_H */
