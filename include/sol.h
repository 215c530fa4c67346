/*
 * sol.h -- C ABI of the MI355X (gfx950) library for the action-conditioned forward pass of a
 * frozen Llama decoder layer (SOL: a per-token discrete "efficiency action" selects an attention
 * keep-rate, an MLP channel keep-rate and an activation bit-width inside the same frozen model).
 *
 * Conventions that hold for every entry point
 *   - Pointers named in a "device" comment are DEVICE pointers (HIP global memory, e.g. a torch
 *     tensor's data_ptr()); structs (sol_model_cfg, sol_action_def[], sol_layer_weights,
 *     sol_model_weights and the per-layer cache pointer arrays) are HOST memory read during the
 *     call only.
 *   - Ownership: every buffer is allocated and owned by the caller. The library borrows it for
 *     the call, never frees it, and allocates device memory only inside sol_create.
 *     Weights are read-only (the base model is frozen; Method, first paragraph).
 *   - Asynchrony: work is enqueued on `stream` (a hipStream_t, NULL = default stream). No entry
 *     point synchronises; outputs are valid once the caller has synchronised the stream.
 *   - Errors: an int status is returned, no exception crosses the ABI; sol_last_error gives text.
 *     Everything that can be checked on the host (null pointers, shapes, table contents,
 *     workspace size, static cache overflow) is checked before the first launch. Conditions that
 *     live in device memory (an action id outside the table, pos0[s] + T > L_max, a token or target
 *     id outside the vocabulary) make the kernels treat the token as a dense-action token / skip the
 *     sequence / clamp the id, and raise a sticky flag that sol_device_status reports.
 *   - Layouts: row-major. Weight matrices are [out_features][in_features]. Activations are
 *     [n_seq][T][d_model]. KV caches are [n_seq][n_kv_heads][L_max][head_dim] with keys stored
 *     after the rotary embedding. Element type of weights, activations and caches is cfg.dtype.
 *   - Determinism: a sequence's outputs do not depend on what else is in the batch, nor on its
 *     slot; no floating-point atomics, no data-dependent reduction order.
 *
 * Numerics with dtype = SOL_BF16: contractions run on bf16 inputs with fp32 accumulation; the
 * tensors handed between operators (normed+quantised linear inputs, q, k, v, attention output,
 * SiLU(gate)*up, layer output) are bf16; the residual inside a layer and all selection /
 * quantisation decisions are fp32. With SOL_F32 everything is fp32.
 */
#ifndef SOL_H
#define SOL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SOL_OK = 0,
    SOL_ERR_INVALID_ARG = -1,   /* null pointer, non-positive size, inconsistent shape          */
    SOL_ERR_UNSUPPORTED = -2,   /* valid request this build has no kernel for                    */
    SOL_ERR_WORKSPACE = -3,     /* workspace pointer null / smaller than sol_workspace_bytes     */
    SOL_ERR_ACTION = -4,        /* action table entry or action id out of range                  */
    SOL_ERR_CACHE_OVERFLOW = -5,/* tokens would be written past L_max                            */
    SOL_ERR_HIP = -6            /* a HIP runtime call failed (text in sol_last_error)            */
} sol_status;

typedef enum { SOL_F32 = 0, SOL_BF16 = 1 } sol_dtype;

/* quant_sites bits: linear-layer inputs that receive the per-token fake-quantiser. */
#define SOL_QS_QKV_IN    1u
#define SOL_QS_O_IN      2u
#define SOL_QS_GATEUP_IN 4u
#define SOL_QS_DOWN_IN   8u
#define SOL_QS_ALL_LINEAR_INPUTS 15u
#define SOL_QS_MLP_OUT   16u  /* output of the MLP block, before the residual add (Appendix
                                 "Activation quantization": the site the paper's own runs use) */

/* One row of the action table a -> (kappa(a), rho(a), q(a)) (Method, "Actions and controlled
 * compute"). Fractions are rationals so that ceil(kappa * n) is exact integer arithmetic.
 * 0 < keep_num <= keep_den, 0 < mlp_keep_num <= mlp_keep_den, bits >= 4; bits >= 16 bypasses
 * the quantiser (Appendix "Quantizer": q >= 16 returns the input unchanged). */
typedef struct {
    uint32_t keep_num, keep_den;          /* kappa: attention keep fraction */
    uint32_t mlp_keep_num, mlp_keep_den;  /* rho:   MLP channel keep fraction */
    uint32_t bits;                        /* q */
} sol_action_def;

typedef struct {
    int32_t d_model, n_q_heads, n_kv_heads, head_dim, d_ff, n_layers, vocab;
    float   rms_eps, rope_theta;
    int32_t dtype;          /* sol_dtype of weights, activations and caches                      */
    int32_t max_positions;  /* rotary table length; every L_max must be <= this                  */
    int32_t page_size;      /* S (Appendix "Quest masking"): 1 = exact per-key top-k; S > 1 =
                               pages of S contiguous keys from key 0, ranked by the upper bound
                               sum_c max(q_c max_c, q_c min_c) over the channel-wise extremes of
                               their allowed keys; the top ceil(b/S) pages are kept whole        */
    int32_t n_sink;         /* T_s: the first n_sink allowed keys are always kept                */
    int32_t n_window;       /* T_w: the last n_window allowed keys are always kept. With S = 1
                               forced keys count against the budget b; with S > 1 they are kept
                               on top of the chosen pages                                        */
    int32_t prune_site;     /* 0 = SiLU(gate)*up intermediate (keep ceil(rho d_ff) channels),
                               1 = MLP input after the post-attention norm (ceil(rho d_model))   */
    uint32_t quant_sites;   /* any subset of SOL_QS_ALL_LINEAR_INPUTS | SOL_QS_MLP_OUT           */
} sol_model_cfg;

typedef struct {  /* device pointers, element type cfg.dtype */
    const void *w_in_norm;   /* [d_model]                         */
    const void *wq;          /* [n_q_heads*head_dim][d_model]     */
    const void *wk;          /* [n_kv_heads*head_dim][d_model]    */
    const void *wv;          /* [n_kv_heads*head_dim][d_model]    */
    const void *wo;          /* [d_model][n_q_heads*head_dim]     */
    const void *w_post_norm; /* [d_model]                         */
    const void *w_gate;      /* [d_ff][d_model]                   */
    const void *w_up;        /* [d_ff][d_model]                   */
    const void *w_down;      /* [d_model][d_ff]                   */
} sol_layer_weights;

typedef struct {
    const void *embed;                /* device [vocab][d_model]; may be NULL if never looked up */
    const sol_layer_weights *layers;  /* host array of cfg.n_layers entries                      */
    const void *w_final_norm;         /* device [d_model]                                        */
    const void *lm_head;              /* device [vocab][d_model]; may alias embed                */
} sol_model_weights;

typedef enum { SOL_OP_LAYER_FORWARD = 0, SOL_OP_DECODE_STEP = 1, SOL_OP_SCHEDULE_LOGLIK = 2, SOL_OP_KV_REFRESH = 3, SOL_OP_REWARD = 4 } sol_op;

typedef struct sol_ctx sol_ctx;

/* Host-only check of a configuration and an action table (no GPU needed).
 * SOL_ERR_ACTION: a table entry violates the ranges above (e.g. kappa = 0, which would leave a
 * softmax over no keys). SOL_ERR_UNSUPPORTED: more than 4096 actions or a head_dim the kernels do
 * not cover. SOL_ERR_INVALID_ARG: bad shape. */
int sol_validate_config(const sol_model_cfg *cfg, const sol_action_def *table, int n_actions);

/* Creates a context on the current HIP device: copies the action table, builds the rotary table
 * (cos/sin of pos * theta^(-2c/head_dim), computed in double on the host) and uploads both.
 * The only entry point that allocates device memory. */
int sol_create(const sol_model_cfg *cfg, const sol_action_def *table, int n_actions, sol_ctx **out);
void sol_destroy(sol_ctx *ctx);
/* Text of the last error on this context (or of the last failed sol_create if ctx is NULL). */
const char *sol_last_error(const sol_ctx *ctx);

/* Bytes of device workspace the operation needs for these sizes (host-only arithmetic).
 * LAYER_FORWARD: (n_seq, T, L_max). DECODE_STEP: (B, ignored, L_max).
 * SCHEDULE_LOGLIK: (B*G, T, ignored). Returns 0 for an invalid request. */
size_t sol_workspace_bytes(const sol_model_cfg *cfg, int op, int n_seq, int T, int L_max);

/* One decoder layer over T tokens per sequence, each under its own action:
 *   input RMSNorm -> [quant] -> q/k/v projections -> rotary -> K/V written to the cache as
 *   computed under the token's action (Background, "Decoding is a stateful process") ->
 *   causal scores over cache positions 0..pos -> keep the ceil(kappa*n) best keys per query head,
 *   ties to the lower position; budget = all keys bypasses selection (Appendix "Token sparsity
 *   via Quest", one key per page) -> softmax over kept keys, times V -> [quant] -> output
 *   projection + residual -> post RMSNorm -> [quant] -> SiLU(gate)*up -> keep the ceil(rho*d_ff)
 *   largest magnitudes per token, ties to the lower channel (Appendix "Structured MLP activation
 *   pruning", operator applied at the intermediate) -> [quant] -> down projection + residual.
 *   [quant] = per-token symmetric fake-quantiser at the token's bit-width (Appendix "Activation
 *   quantization") at the sites enabled in cfg.quant_sites.
 * x_in, x_out: device [n_seq][T][d_model] (may not alias). action_ids: device int32 [n_seq][T].
 * pos0: device int32 [n_seq], tokens already in each sequence's cache (NULL = all zero); token i
 * sits at position pos0[s]+i. k_cache, v_cache: device, read at [0,pos] and written at
 * [pos0, pos0+T). workspace: device, >= sol_workspace_bytes(cfg, SOL_OP_LAYER_FORWARD, ...). */
int sol_layer_forward(sol_ctx *ctx, const sol_layer_weights *w, const void *x_in, void *x_out,
                      const int32_t *action_ids, const int32_t *pos0,
                      void *k_cache, void *v_cache, int n_seq, int T, int L_max,
                      void *workspace, size_t ws_bytes, void *stream);

/* One token per sequence through all cfg.n_layers layers (the decode step). The token's K/V are
 * appended at cache_len[s] in every layer. Input is token_ids (device int32 [B], looked up in
 * weights->embed) or, if token_ids is NULL, x_in (device [B][d_model]). action_ids, cache_len:
 * device int32 [B]. k_cache, v_cache: host arrays of n_layers device pointers.
 * x_out: device [B][d_model], the last layer's output (before the final norm); may be NULL.
 * If nll_out (device float [B]) is non-NULL, targets (device int32 [B]) is required and
 * nll_out[s] = logsumexp(W_lm hf) - (W_lm hf)[target], hf = final RMSNorm (Method, Eq. 1). */
int sol_decode_step(sol_ctx *ctx, const sol_model_weights *weights,
                    const int32_t *token_ids, const void *x_in,
                    const int32_t *action_ids, const int32_t *cache_len,
                    void *const *k_cache, void *const *v_cache, int B, int L_max,
                    void *x_out, const int32_t *targets, float *nll_out,
                    void *workspace, size_t ws_bytes, void *stream);

/* sol_decode_step for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc. Same arguments, results and error behaviour as
 * sol_decode_step, bit for bit, without the workspace: the step's scratch (K-split partial sums, the row plan,
 * activations between the kernels, a chunk of logits) lives in a file-scope device array of
 * sol_static_scratch_bytes() = 64 MiB that every GPU the library runs on holds until the process ends. The call
 * allocates and frees nothing. A step whose sol_workspace_bytes(cfg, SOL_OP_DECODE_STEP, B, 1, L_max) exceeds that
 * size is rejected with SOL_ERR_WORKSPACE before any launch (64 sequences of the Llama-3.2-1B shape need 51 MiB).
 * The context must have been created on the device that is current at the call (SOL_ERR_INVALID_ARG otherwise).
 * Every call on a GPU shares that GPU's one array: calls that overlap on one GPU (two streams, two contexts, two
 * threads) race on it; the array keeps the last call's contents and nothing in it needs clearing between calls
 * (every kernel of the step writes what it later reads). */
size_t sol_static_scratch_bytes(void);
int sol_decode_step_static(sol_ctx *ctx, const sol_model_weights *weights,
                           const int32_t *token_ids, const void *x_in,
                           const int32_t *action_ids, const int32_t *cache_len,
                           void *const *k_cache, void *const *v_cache, int B, int L_max,
                           void *x_out, const int32_t *targets, float *nll_out, void *stream);

/* Page metadata for decoding under the page rule (cfg.page_size = S >= 2; Appendix "Quest masking": the
 * element-wise maximum and minimum of the keys of each page). One buffer per layer, device memory owned by
 * the caller, sol_page_meta_bytes(cfg, n_seq, L_max) bytes, laid out
 * [n_seq][n_kv_heads][ceil(L_max / S)][2 * head_dim] of cfg.dtype: per page the channel-wise maxima followed
 * by the minima of the keys written so far. With it a decode step reads 2 / S of the key cache for the page
 * bounds plus the pages it keeps, instead of every key. bf16, head_dim 64 or 128, 4 query heads per KV head;
 * anything else: SOL_ERR_UNSUPPORTED (sol_decode_step itself handles every configuration, reading all keys).
 *
 * sol_page_meta_build: metadata of keys [0, cache_len[s]) of one layer's key cache (device
 * [n_seq][n_kv_heads][L_max][head_dim]); pages past cache_len[s] are left untouched.
 * sol_decode_step_paged: sol_decode_step with page_meta, a host array of n_layers device pointers; the
 * new token's key is folded into its page in every layer, so the same buffers serve the next step. */
size_t sol_page_meta_bytes(const sol_model_cfg *cfg, int n_seq, int L_max);
int sol_page_meta_build(sol_ctx *ctx, const void *k_cache, const int32_t *cache_len, int n_seq, int L_max,
                        void *page_meta, void *stream);
int sol_decode_step_paged(sol_ctx *ctx, const sol_model_weights *weights,
                          const int32_t *token_ids, const void *x_in,
                          const int32_t *action_ids, const int32_t *cache_len,
                          void *const *k_cache, void *const *v_cache, void *const *page_meta, int B, int L_max,
                          void *x_out, const int32_t *targets, float *nll_out,
                          void *workspace, size_t ws_bytes, void *stream);

/* Periodic KV-cache refresh (Background, "Episodes and control horizon"): a fully dense pass of all
 * cfg.n_layers layers over the T already-known tokens of every sequence, token i of sequence s at position
 * pos0[s] + i, attending to the cache before it; their K/V entries in every layer are overwritten with the dense
 * values (every key kept, no pruning, every quantiser bypassed, whatever cfg says). Nothing is sampled.
 * Input: token_ids (device int32 [n_seq][T], looked up in weights->embed) or, if NULL, x_in (device
 * [n_seq][T][d_model]). pos0: device int32 [n_seq]; pos0[s] + T > L_max sets the cache-overflow flag and skips
 * the sequence. k_cache, v_cache: host arrays of n_layers device pointers. page_meta: NULL, or the per-layer
 * page metadata buffers, whose pages holding rewritten keys are rebuilt. x_out: device [n_seq][T][d_model], the
 * last layer's output, may be NULL. Workspace: sol_workspace_bytes(cfg, SOL_OP_KV_REFRESH, n_seq, T, L_max).
 * n_seq * T == 0 is a no-op. */
int sol_kv_refresh(sol_ctx *ctx, const sol_model_weights *weights,
                   const int32_t *token_ids, const void *x_in, const int32_t *pos0,
                   void *const *k_cache, void *const *v_cache, void *const *page_meta,
                   int n_seq, int T, int L_max, void *x_out,
                   void *workspace, size_t ws_bytes, void *stream);

/* Episode pass (Method, "GRPO with per-sequence budget sampling"): for every input a dense prefill of its P-token
 * context prefix, run once, initialises the cache; K counterfactual schedules of T teacher-forced steps then share
 * that prefix and the token path and differ only in their actions:
 *   nll_out[b][k][t] = -log p(targets[b][t]) of step t of schedule k, the token at position P + t attending to the
 *   dense prefix and to the schedule's own earlier steps, under action_ids[b][k][t].
 * It equals sol_schedule_loglik on the P + T tokens with the dense action on the prefix, restricted to the last T
 * positions, without running the prefix K times. prefix_tokens: device int32 [B][P]; tokens, targets: device int32
 * [B][T]; action_ids: device int32 [B][K][T]; nll_out: device float [B][K][T]. The prefix is dense whatever cfg
 * says. Workspace: sol_episode_workspace_bytes(cfg, B, K, P, T) (holds one layer's caches for B * K sequences).
 * B * K * T == 0 is a no-op; P must be positive. The K schedules of an input read its prefix cache in place when
 * the tiled attention kernels cover the shape (bf16, page_size 1 without sink / window keys, P a multiple of 64,
 * T >= 16, P + T <= 4096, or the page rule with P a multiple of 16 pages); otherwise each schedule works on a
 * copy, with the same results bit for bit (sol_test_episode_loglik_copies below forces the copies). */
size_t sol_episode_workspace_bytes(const sol_model_cfg *cfg, int B, int K, int P, int T);
int sol_episode_loglik(sol_ctx *ctx, const sol_model_weights *weights, const int32_t *prefix_tokens,
                       const int32_t *tokens, const int32_t *targets, const int32_t *action_ids,
                       int B, int K, int P, int T, float *nll_out,
                       void *workspace, size_t ws_bytes, void *stream);

/* Reward reduction on the output of sol_schedule_loglik (Method, "Actions and controlled compute", Eqs. 2-5;
 * "GRPO with per-sequence budget sampling"). With r_t = -nll[b][g][t] the task reward of step t:
 *   avg[b][g]     = (kappa, rho, eta = min(q, 16) / 16) of the schedule's actions averaged over its effective steps
 *                   (eff[b][t] != 0; eff NULL = every step; no effective step: the targets, so no penalty);
 *   penalty[b][g] = sum over the three axes of alpha * max(0, |avg - target| - tau)^2      (Eq. 3)
 *   returns       = G_t = sum_{u >= t} gamma^(u - t) r_u                                  (Eq. 4)
 *   signal        = G_t - penalty[b][g]                                                   (Eq. 5)
 *   adv           = signal minus its mean over the G schedules of input b at the same t, then whitened over all
 *                   B * G * T values: (x - mean) / (population std + eps).
 * nll, action_ids: device [B][G][T] (float / int32); eff: device int32 [B][T] or NULL; targets: device float
 * [B][3] = (C_kappa, C_rho, C_eta) per input. Outputs are device float arrays: avg_out [B][G][3], penalty_out
 * [B][G], returns_out [B][G][T] (each may be NULL), signal_out and adv_out [B][G][T] (required; they must not
 * alias nll). An action id outside the table counts as action 0 and sets the bad-action flag.
 * Workspace: sol_workspace_bytes(cfg, SOL_OP_REWARD, B, T, 0) bytes. B * G * T == 0 is a no-op. */
typedef struct {
    float alpha_kappa, alpha_rho, alpha_eta;  /* trade-off weights, >= 0                     */
    float tau;                                /* tolerance band, >= 0                        */
    float gamma;                              /* discount in (0, 1]                          */
    float eps;                                /* added to the standard deviation, >= 0       */
} sol_reward_cfg;
int sol_reward_advantages(sol_ctx *ctx, const float *nll, const int32_t *action_ids, const int32_t *eff,
                          const float *targets, const sol_reward_cfg *rc, int B, int G, int T,
                          float *avg_out, float *penalty_out, float *returns_out, float *signal_out, float *adv_out,
                          void *workspace, size_t ws_bytes, void *stream);

/* Teacher-forced pass over G compute schedules that share one token path (Method, "GRPO with
 * per-sequence budget sampling"): for every input b, schedule g and position t,
 *   nll_out[b][g][t] = -log p_t^{a}(targets[b][t])  in nats (Method, Eq. 1, negated),
 * the full stack run under action_ids[b][g][.] with the same action in every layer of a step.
 * tokens, targets: device int32 [B][T]; action_ids: device int32 [B][G][T];
 * nll_out: device float [B][G][T]. KV caches live in the workspace. */
int sol_schedule_loglik(sol_ctx *ctx, const sol_model_weights *weights,
                        const int32_t *tokens, const int32_t *targets, const int32_t *action_ids,
                        int B, int G, int T, float *nll_out,
                        void *workspace, size_t ws_bytes, void *stream);

/* Synchronises `stream`, returns and clears the sticky device flags:
 * SOL_OK, SOL_ERR_CACHE_OVERFLOW (a sequence was skipped because pos0 + T > L_max), SOL_ERR_ACTION (an action id
 * outside the table was met and treated as dense) or SOL_ERR_INVALID_ARG (a token id or a target id outside
 * [0, vocab) was met and clamped into it: the embedding lookups and the NLLs of sol_schedule_loglik,
 * sol_episode_loglik, sol_decode_step and sol_kv_refresh of that call are then those of the clamped ids). */
int sol_device_status(sol_ctx *ctx, void *stream);

/* Per-stage timing for measurement. sol_profile_enable(ctx, n) with n > 0 creates up to n pairs of
 * HIP events and makes every following call bracket each stage of the path (one stage = the
 * kernel(s) of one step: qkv_gemm, attention_topk, gate_up_gemm, ...) with events on the caller's
 * stream; n <= 0 switches it off. sol_profile_read synchronises `stream`, writes for each stage its
 * name (static string), the summed milliseconds and the number of recorded brackets since the last
 * read into the caller's HOST arrays of max_stages entries, clears the records and returns the
 * number of stages written (or a negative status). Records beyond n are dropped silently. */
int sol_profile_enable(sol_ctx *ctx, int max_stage_records);
int sol_profile_read(sol_ctx *ctx, void *stream, int max_stages, const char **names_out, float *ms_out,
                     int *calls_out);

/* Measured peaks of the GPU the library runs on, for pricing rooflines beside the published figures: a register-only
 * loop of bf16 32x32x16 MFMAs on every SIMD (TFLOP/s), a plain device copy of half of `scratch` into its other half
 * (GB/s, bytes read plus bytes written) and a read-only sweep of that half (GB/s). scratch: device memory the caller
 * owns, at least 64 MiB, best 2 GiB or more so that the sweeps do not live in the memory-side cache. `reps` launches
 * of each are timed with events on `stream`; the call synchronises. Returns SOL_OK, SOL_ERR_INVALID_ARG,
 * SOL_ERR_WORKSPACE (scratch too small) or SOL_ERR_HIP. */
int sol_measure_peaks(void *scratch, size_t scratch_bytes, int reps, float *mfma_tflops_out, float *copy_gbs_out,
                      float *read_gbs_out, void *stream);

/* ---- unit hooks: the selection / quantisation device code on caller-supplied fp32 data ----
 * All pointers device; results are exact integer decisions and must match the definitions
 * bit for bit. */

/* Row r holds n_cols fp32 scores of which the first n_valid[r] are allowed; keep_out[r][j] = 1
 * for the k[r] largest allowed scores (ties to the lower j), 0 elsewhere. 1 <= k[r] <= n_valid[r]. */
int sol_test_topk_select(const float *scores, int rows, int n_cols, const int32_t *n_valid,
                         const int32_t *k, uint8_t *keep_out, void *stream);
/* The same decision taken by the row stage of the batched attention path (Method, "Actions and controlled
 * execution", attention keep-rate: the budget's largest causal scores of a query, ties to the earlier key): fp32 score rows go through the
 * key transform, threshold search and tie index of the threshold kernel, and keep_out is what the
 * softmax kernel would keep from {threshold, tie index}. Arguments as sol_test_topk_select;
 * n_cols <= 4096 (the longest row of the batched path), else SOL_ERR_UNSUPPORTED and nothing is written. */
int sol_test_attn_threshold(const float *scores, int rows, int n_cols, const int32_t *n_valid,
                            const int32_t *k, uint8_t *keep_out, void *stream);
/* keep_out[r][c] = 1 for the m[r] largest |a[r][c]| (ties to the lower c). */
int sol_test_prune_mask(const float *a, int rows, int n, const int32_t *m, uint8_t *keep_out,
                        void *stream);
/* The production "magnitude pruning + fake-quantise" kernel (the down-projection input step of the
 * layer) in place on caller rows a[r][0..n) of element type dtype: keeps the m[r] largest |a|, ties
 * to the lower channel, zeroes the rest, then quantises at bits[r] (>= 16: no quantiser) and rounds
 * to dtype. scratch: device, >= 16 * rows bytes. n * 4 bytes must fit 60 KB of LDS. */
int sol_test_prune_quant(void *a, int dtype, int rows, int n, const int32_t *m, const int32_t *bits,
                         void *scratch, size_t scratch_bytes, void *stream);
/* Per-row fake-quantiser: codes_out[r][j] (int32), scale_out[r], dequantised z_hat_out[r][j].
 * bits[r] >= 16: codes 0, scale 0, z_hat = z. */
int sol_test_quant_codes(const float *z, int rows, int n, const int32_t *bits,
                         int32_t *codes_out, float *scale_out, float *zhat_out, void *stream);

/* The layer's bf16 MFMA GEMM on caller data: c[M][N] (fp32) = a[M][K] (bf16) * w[N][K]^T (bf16), fp32
 * accumulation: the product behind every linear map of the frozen layer (the paper takes the Llama block as
 * given; Appendix "Structured MLP activation pruning" writes the MLP as such products). N a multiple of
 * 256 and K a multiple of 128, else SOL_ERR_UNSUPPORTED; M >= 0 (ragged last tile allowed). */
int sol_test_gemm(const void *a, const void *w, float *c, int M, int N, int K, void *stream);

/* ---- stage hooks: one stage of sol_layer_forward on caller-supplied operands, through the same dispatch and
 * kernels as the layer, so that a comparison with a reference crosses at most one quantiser. Workspace:
 * sol_workspace_bytes(cfg, SOL_OP_LAYER_FORWARD, n_seq, T, L_max). */

/* Attention stage (Appendix "Token sparsity via Quest"): q device [n_seq][T][n_q_heads*head_dim] of cfg.dtype,
 * queries after the rotary embedding; k_cache / v_cache as in sol_layer_forward, already holding the keys and
 * values of positions [0, pos0[s] + T); token i of sequence s attends positions [0, pos0[s] + i] under
 * action_ids[s][i] and cfg's selection rule. o_out: device float [n_seq][T][n_q_heads*head_dim], the attention
 * output before the quantiser of the output projection's input. */
int sol_test_attention_stage(sol_ctx *ctx, const void *q, const int32_t *action_ids, const int32_t *pos0,
                             void *k_cache, void *v_cache, int n_seq, int T, int L_max, float *o_out,
                             void *workspace, size_t ws_bytes, void *stream);

/* MLP stage (Appendix "Structured MLP activation pruning", "Activation quantization"): h2 device [n_seq][T][d_model]
 * of cfg.dtype, the MLP input as the gate / up projections read it (after norm, MLP-input pruning and its quantiser);
 * x2 device float [n_seq][T][d_model], the residual after attention. Runs gate / up, SiLU(gate)*up, magnitude pruning
 * and the quantiser of the down projection's input, the down projection, the MLP-output quantiser if enabled, and
 * the residual add. a_out: NULL or device [n_seq][T][d_ff] of cfg.dtype, the down projection's input; x_out: device
 * [n_seq][T][d_model] of cfg.dtype. Workspace sized with L_max = T. */
int sol_test_mlp_stage(sol_ctx *ctx, const sol_layer_weights *w, const void *h2, const float *x2,
                       const int32_t *action_ids, int n_seq, int T, void *a_out, void *x_out,
                       void *workspace, size_t ws_bytes, void *stream);

/* sol_episode_loglik with every schedule working on its own copy of the prefix cache, whatever the shape (the
 * fall-back layout of that entry point); workspace sized by sol_test_episode_copies_workspace_bytes. The results
 * equal sol_episode_loglik's bit for bit. */
size_t sol_test_episode_copies_workspace_bytes(const sol_model_cfg *cfg, int B, int K, int P, int T);
int sol_test_episode_loglik_copies(sol_ctx *ctx, const sol_model_weights *weights, const int32_t *prefix_tokens,
                                   const int32_t *tokens, const int32_t *targets, const int32_t *action_ids,
                                   int B, int K, int P, int T, float *nll_out,
                                   void *workspace, size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif
