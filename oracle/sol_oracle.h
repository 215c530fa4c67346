/*
 * sol_oracle.h -- CPU oracle for the action-conditioned forward pass of a frozen
 * Llama decoder layer (SOL, "Compute Where it Counts").
 *
 * THIS IS TEST INFRASTRUCTURE. It is a plain, slow, obviously-correct
 * implementation that the GPU library is checked against. It shares no code,
 * header, table or helper with the HIP path and the product never calls it.
 * Only the tests, the smoke check and the benchmark's cpu_baseline leg load it.
 *
 * Numerics: fp32 storage, every dot product / sum accumulated in fp64 in index
 * order; the fake-quantiser is evaluated in fp32 IEEE arithmetic exactly as the
 * paper's formula is written (Appendix "Activation quantization").
 *
 * All pointers are HOST pointers to float32 / int32 data owned by the caller.
 * Weight matrices are row-major [out_features][in_features].
 * KV caches are [n_seq][n_kv_heads][L_max][head_dim] float32, keys stored after
 * the rotary embedding.
 *
 * Pins (tests/test_oracle_*.py): dense special case against PyTorch CPU
 * primitives; brute-force rank selection on tiny inputs; closed forms for the
 * quantiser, the page bound, softmax and NLL; batched == step-wise; causality;
 * the bf16-store mode against a float64 witness that rounds through
 * torch.bfloat16 at exactly the hand-over points (and must disagree when any
 * one of them is left out); the page rule inside the layer against a numpy
 * page ranking on the witness's own q and k.
 * No value printed by the paper exists for any operator (the paper gives no
 * worked numeric example), so against the paper's own numbers parity is
 * unpinned; the invariants above are the whole net.
 */
#ifndef SOL_ORACLE_H
#define SOL_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* quant_sites bits: where the per-token fake-quantiser is applied. */
#define ORC_QS_QKV_IN   1u   /* input of q/k/v projections (after input norm)  */
#define ORC_QS_O_IN     2u   /* input of the output projection                 */
#define ORC_QS_GATEUP_IN 4u  /* input of gate/up projections (after post norm) */
#define ORC_QS_DOWN_IN  8u   /* input of the down projection (after pruning)   */
#define ORC_QS_MLP_OUT  16u  /* output of the MLP block (the paper's own site) */

typedef struct {
    int32_t d_model, n_q_heads, n_kv_heads, head_dim, d_ff, n_layers, vocab;
    float   rms_eps, rope_theta;
    int32_t page_size;   /* S: 1 = exact per-key top-k; >1 = Quest page bound   */
    int32_t n_sink;      /* first keys always kept  (T_s)                        */
    int32_t n_window;    /* last keys always kept   (T_w)                        */
    int32_t prune_site;  /* 0 = SiLU(gate)*up intermediate, 1 = MLP input        */
    uint32_t quant_sites;
    int32_t act_bf16;    /* 1: tensors handed between operators are rounded to
                            bfloat16 (h1, q, k, v, o, h2, a, layer output);
                            0: everything stays fp32                              */
} orc_cfg;

typedef struct {
    uint32_t keep_num, keep_den;         /* kappa = attention keep fraction     */
    uint32_t mlp_keep_num, mlp_keep_den; /* rho   = MLP channel keep fraction   */
    uint32_t bits;                       /* q; >= 16 means bypass               */
} orc_action;

typedef struct {
    const float *w_in_norm, *wq, *wk, *wv, *wo, *w_post_norm, *w_gate, *w_up, *w_down;
} orc_layer_weights;

/* ---- single operators (each is also a unit under test) ------------------ */

/* b = ceil(num * n / den) in integers, clamped to [1, n].
 * Appendix "Budgeted token selection": b_t = ceil(kappa_t * K_t). */
int32_t orc_budget(uint32_t num, uint32_t den, int32_t n);

/* Per-token symmetric fake-quantiser (Appendix "Quantizer").
 * out may alias z. codes/scale may be NULL. bits >= 16: copy, codes = 0. */
void orc_fake_quant(const float *z, int32_t n, int32_t bits,
                    float *out, int32_t *codes, float *scale);

/* keep[c] = 1 for the m entries of largest |a[c]| (ties: lower c wins).
 * Appendix "Per-token channel selection". */
void orc_topm_mask(const float *a, int32_t n, int32_t m, uint8_t *keep);

/* Page size 1: keep[j] = 1 for forced keys (first n_sink, last n_window of the
 * n allowed keys) and the best-scoring others until b keys are kept
 * (ties: lower j wins). Appendix "Quest masking", one key per page. */
void orc_select_keys(const float *score, int32_t n, int32_t b,
                     int32_t n_sink, int32_t n_window, uint8_t *keep);

/* Quest page bound (Appendix "Quest masking"): pages of S contiguous keys
 * starting at key 0; page score = q_pos . m_plus + q_neg . m_minus over the
 * page's allowed keys; keep the top ceil(b/S) pages (ties: lower page wins)
 * plus the forced keys. k_rows points at key 0, consecutive keys k_stride
 * floats apart. page_score_out (ceil(n/S) floats) may be NULL. */
void orc_select_pages(const float *q, const float *k_rows, int64_t k_stride,
                      int32_t head_dim, int32_t n, int32_t b, int32_t S,
                      int32_t n_sink, int32_t n_window,
                      uint8_t *keep, float *page_score_out);

/* softmax over the kept keys of the scaled scores, times V.
 * prob_out (n floats, 0 for dropped keys) may be NULL. */
void orc_softmax_v(const float *score, const uint8_t *keep, int32_t n,
                   const float *v_rows, int64_t v_stride, int32_t head_dim,
                   float *o, float *prob_out);

/* nll = logsumexp_v(w_lm[v] . hf) - w_lm[target] . hf   (Eq. 1, negated). */
float orc_nll_row(const float *hf, const float *w_lm, int32_t d, int32_t vocab,
                  int32_t target);

/* RMSNorm of one row: out = x * rsqrt(mean(x^2) + eps) * w. */
void orc_rmsnorm(const float *x, const float *w, int32_t d, float eps, float *out);

/* round-to-nearest-even to bfloat16, returned widened to float. */
float orc_round_bf16(float x);

/* ---- the path ------------------------------------------------------------ */

/* Optional taps, all may be NULL. keep_mask: [n_seq][T][n_q_heads][L_max] bytes,
 * entry 1 where the key was attended. */
typedef struct {
    uint8_t *keep_mask;
    float   *attn_out;   /* [n_seq*T][n_q_heads*head_dim], before site B      */
    float   *mlp_act;    /* [n_seq*T][d_ff], after prune + site D             */
    float   *x_mid;      /* [n_seq*T][d_model], residual after attention      */
    float   *q_rot;      /* [n_seq*T][n_q_heads*head_dim], queries after the
                            rotary embedding, as attention reads them         */
    float   *h2;         /* [n_seq*T][d_model], MLP input as the gate / up
                            projections read it (after norm, prune, site C)   */
    float   *h1;         /* [n_seq*T][d_model], input of the q/k/v projections
                            (after the input norm and site A)                 */
} orc_taps;

/* One decoder layer over T tokens per sequence. Token i of sequence s sits at
 * absolute position pos0[s] + i (pos0 == NULL: 0) and runs under
 * table[action_ids[s*T+i]]; its K/V are written to the cache as computed.
 * Returns 0, or a negative code: -1 bad argument, -4 bad action, -5 cache
 * overflow. */
int32_t orc_layer_forward(const orc_cfg *cfg, const orc_action *table, int32_t n_actions,
                          const orc_layer_weights *w,
                          const float *x_in, float *x_out,
                          const int32_t *action_ids, const int32_t *pos0,
                          float *k_cache, float *v_cache,
                          int32_t n_seq, int32_t T, int32_t L_max,
                          const orc_taps *taps);

/* One token per sequence through all layers. x0 is [B][d_model] (the embedded
 * token). k_cache[l], v_cache[l] are the per-layer caches. The new K/V are
 * written at cache_len[s]. hidden_out [B][d_model] (before the final norm) and
 * nll_out [B] (needs w_final_norm, lm_head, targets) may be NULL. */
int32_t orc_decode_step(const orc_cfg *cfg, const orc_action *table, int32_t n_actions,
                        const orc_layer_weights *layers,
                        const float *w_final_norm, const float *lm_head,
                        const float *x0, const int32_t *action_ids,
                        const int32_t *cache_len,
                        float *const *k_cache, float *const *v_cache,
                        int32_t B, int32_t L_max,
                        float *hidden_out, const int32_t *targets, float *nll_out);

/* Full stack, G schedules over the same token path. tokens/targets [B][T],
 * action_ids [B][G][T], nll_out [B][G][T] in nats. hidden_out (may be NULL) is
 * [B][G][T][d_model], the last layer's output before the final norm. */
int32_t orc_schedule_loglik(const orc_cfg *cfg, const orc_action *table, int32_t n_actions,
                            const float *embed, const orc_layer_weights *layers,
                            const float *w_final_norm, const float *lm_head,
                            const int32_t *tokens, const int32_t *targets,
                            const int32_t *action_ids,
                            int32_t B, int32_t G, int32_t T,
                            float *nll_out, float *hidden_out);

/* threads the parallel loops will use */
int32_t orc_num_threads(void);

#ifdef __cplusplus
}
#endif
#endif
