/*
 * sol_oracle.c -- CPU oracle (test infrastructure; see sol_oracle.h).
 *
 * Written from the paper's operator definitions, one loop per formula:
 *   - budget, page bound, additive -inf mask  : Appendix "Token sparsity via Quest"
 *   - per-token magnitude top-m channel mask  : Appendix "Structured MLP activation pruning"
 *   - symmetric per-token fake-quantiser      : Appendix "Activation quantization"
 *   - per-step task reward = token log-lik    : Method, Eq. (1)
 *   - K/V committed as computed under action  : Background, "Decoding is a stateful process"
 * around a textbook Llama decoder block (RMSNorm, rotary embedding in the
 * rotate-half convention, grouped-query causal attention, SwiGLU MLP).
 *
 * fp32 storage, fp64 accumulation in index order. No blocking, no fusion.
 * OpenMP only across independent rows / heads.
 */
#include "sol_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int32_t orc_num_threads(void)
{
#ifdef _OPENMP
    return (int32_t)omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------ */
/* small helpers                                                             */
/* ------------------------------------------------------------------------ */

float orc_round_bf16(float x)
{
    uint32_t u;
    memcpy(&u, &x, 4);
    if ((u & 0x7F800000u) == 0x7F800000u) {      /* inf / nan: truncate, keep nan */
        if (u & 0x007FFFFFu) u |= 0x00400000u;
        u &= 0xFFFF0000u;
    } else {
        u += 0x7FFFu + ((u >> 16) & 1u);         /* round to nearest, ties to even */
        u &= 0xFFFF0000u;
    }
    memcpy(&x, &u, 4);
    return x;
}

static void round_row(float *x, int32_t n, int32_t act_bf16)
{
    if (!act_bf16) return;
    for (int32_t i = 0; i < n; ++i) x[i] = orc_round_bf16(x[i]);
}

static double dot64(const float *a, const float *b, int32_t n)
{
    double acc = 0.0;
    for (int32_t i = 0; i < n; ++i) acc += (double)a[i] * (double)b[i];
    return acc;
}

/* y[o] = sum_i W[o][i] x[i], W row-major [n_out][n_in] */
static void matvec(const float *W, const float *x, int32_t n_out, int32_t n_in, float *y)
{
    for (int32_t o = 0; o < n_out; ++o)
        y[o] = (float)dot64(W + (int64_t)o * n_in, x, n_in);
}

int32_t orc_budget(uint32_t num, uint32_t den, int32_t n)
{
    if (n <= 0) return 0;
    uint64_t b = ((uint64_t)num * (uint64_t)n + (uint64_t)den - 1u) / (uint64_t)den;
    if (b < 1u) b = 1u;
    if (b > (uint64_t)n) b = (uint64_t)n;
    return (int32_t)b;
}

void orc_rmsnorm(const float *x, const float *w, int32_t d, float eps, float *out)
{
    double ss = 0.0;
    for (int32_t j = 0; j < d; ++j) ss += (double)x[j] * (double)x[j];
    double r = 1.0 / sqrt(ss / (double)d + (double)eps);
    for (int32_t j = 0; j < d; ++j) out[j] = (float)((double)x[j] * r * (double)w[j]);
}

/* ------------------------------------------------------------------------ */
/* fake-quantiser: q_max = 2^(b-1)-1, a = max|z|, s = a/q_max,               */
/* z_hat = clip(round(z/s), -q_max, q_max) * s ; b >= 16 returns z.          */
/* Evaluated in fp32, round half to even.                                    */
/* ------------------------------------------------------------------------ */
void orc_fake_quant(const float *z, int32_t n, int32_t bits,
                    float *out, int32_t *codes, float *scale)
{
    if (bits >= 16) {
        for (int32_t j = 0; j < n; ++j) { if (codes) codes[j] = 0; out[j] = z[j]; }
        if (scale) *scale = 0.0f;
        return;
    }
    const float q_max = (float)((1 << (bits - 1)) - 1);
    float a = 0.0f;
    for (int32_t j = 0; j < n; ++j) { float m = fabsf(z[j]); if (m > a) a = m; }
    if (a == 0.0f) {                               /* all-zero row: unchanged */
        for (int32_t j = 0; j < n; ++j) { if (codes) codes[j] = 0; out[j] = z[j]; }
        if (scale) *scale = 0.0f;
        return;
    }
    const float s = a / q_max;                     /* fp32 IEEE divide */
    if (scale) *scale = s;
    for (int32_t j = 0; j < n; ++j) {
        const float t = z[j] / s;                  /* fp32 IEEE divide */
        float c = rintf(t);                        /* ties to even (default mode) */
        if (c >  q_max) c =  q_max;
        if (c < -q_max) c = -q_max;
        if (codes) codes[j] = (int32_t)c;
        out[j] = c * s;
    }
}

/* ------------------------------------------------------------------------ */
/* magnitude / score selection via a full sort (descending key, ascending    */
/* index among equals)                                                        */
/* ------------------------------------------------------------------------ */
typedef struct { float key; int32_t idx; } keyed;

static int cmp_desc_key_asc_idx(const void *pa, const void *pb)
{
    const keyed *a = (const keyed *)pa, *b = (const keyed *)pb;
    if (a->key > b->key) return -1;
    if (a->key < b->key) return 1;
    return (a->idx > b->idx) - (a->idx < b->idx);
}

void orc_topm_mask(const float *a, int32_t n, int32_t m, uint8_t *keep)
{
    memset(keep, 0, (size_t)n);
    if (m <= 0) return;
    if (m >= n) { memset(keep, 1, (size_t)n); return; }
    keyed *v = (keyed *)malloc(sizeof(keyed) * (size_t)n);
    for (int32_t c = 0; c < n; ++c) { v[c].key = fabsf(a[c]); v[c].idx = c; }
    qsort(v, (size_t)n, sizeof(keyed), cmp_desc_key_asc_idx);
    for (int32_t r = 0; r < m; ++r) keep[v[r].idx] = 1;
    free(v);
}

static int32_t mark_forced(int32_t n, int32_t n_sink, int32_t n_window, uint8_t *keep)
{
    int32_t forced = 0;
    for (int32_t j = 0; j < n; ++j) {
        int f = (j < n_sink) || (j >= n - n_window);
        keep[j] = (uint8_t)f;
        forced += f;
    }
    return forced;
}

void orc_select_keys(const float *score, int32_t n, int32_t b,
                     int32_t n_sink, int32_t n_window, uint8_t *keep)
{
    if (n <= 0) return;
    if (b >= n) { memset(keep, 1, (size_t)n); return; }
    int32_t forced = mark_forced(n, n_sink, n_window, keep);
    int32_t rest = b - forced;
    if (rest <= 0) return;
    keyed *v = (keyed *)malloc(sizeof(keyed) * (size_t)n);
    int32_t cnt = 0;
    for (int32_t j = 0; j < n; ++j)
        if (!keep[j]) { v[cnt].key = score[j]; v[cnt].idx = j; ++cnt; }
    qsort(v, (size_t)cnt, sizeof(keyed), cmp_desc_key_asc_idx);
    for (int32_t r = 0; r < rest && r < cnt; ++r) keep[v[r].idx] = 1;
    free(v);
}

void orc_select_pages(const float *q, const float *k_rows, int64_t k_stride,
                      int32_t head_dim, int32_t n, int32_t b, int32_t S,
                      int32_t n_sink, int32_t n_window,
                      uint8_t *keep, float *page_score_out)
{
    if (n <= 0) return;
    const int32_t n_pages = (n + S - 1) / S;
    keyed *pg = (keyed *)malloc(sizeof(keyed) * (size_t)n_pages);
    for (int32_t u = 0; u < n_pages; ++u) {
        const int32_t j0 = u * S;
        const int32_t j1 = (j0 + S < n) ? j0 + S : n;      /* allowed keys only */
        double sc = 0.0;
        for (int32_t c = 0; c < head_dim; ++c) {
            float mx = k_rows[(int64_t)j0 * k_stride + c];
            float mn = mx;
            for (int32_t j = j0 + 1; j < j1; ++j) {
                float kv = k_rows[(int64_t)j * k_stride + c];
                if (kv > mx) mx = kv;
                if (kv < mn) mn = kv;
            }
            const double m_plus = (double)mx, m_minus = -(double)mn;
            const double qa = fabs((double)q[c]);
            const double q_pos = (q[c] >= 0.0f) ? qa : 0.0;
            const double q_neg = qa - q_pos;
            sc += q_pos * m_plus + q_neg * m_minus;
        }
        pg[u].key = (float)sc;
        pg[u].idx = u;
        if (page_score_out) page_score_out[u] = (float)sc;
    }
    if (b >= n) { memset(keep, 1, (size_t)n); free(pg); return; }
    mark_forced(n, n_sink, n_window, keep);
    int32_t n_keep_pages = (b + S - 1) / S;
    if (n_keep_pages > n_pages) n_keep_pages = n_pages;
    qsort(pg, (size_t)n_pages, sizeof(keyed), cmp_desc_key_asc_idx);
    for (int32_t r = 0; r < n_keep_pages; ++r) {
        const int32_t j0 = pg[r].idx * S;
        const int32_t j1 = (j0 + S < n) ? j0 + S : n;
        for (int32_t j = j0; j < j1; ++j) keep[j] = 1;
    }
    free(pg);
}

void orc_softmax_v(const float *score, const uint8_t *keep, int32_t n,
                   const float *v_rows, int64_t v_stride, int32_t head_dim,
                   float *o, float *prob_out)
{
    double *p = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
    double mx = -INFINITY;
    for (int32_t j = 0; j < n; ++j) if (keep[j] && (double)score[j] > mx) mx = (double)score[j];
    double den = 0.0;
    for (int32_t j = 0; j < n; ++j) {
        p[j] = keep[j] ? exp((double)score[j] - mx) : 0.0;   /* dropped key: exp(-inf) = 0 */
        den += p[j];
    }
    for (int32_t j = 0; j < n; ++j) p[j] /= den;
    for (int32_t c = 0; c < head_dim; ++c) {
        double acc = 0.0;
        for (int32_t j = 0; j < n; ++j)
            if (keep[j]) acc += p[j] * (double)v_rows[(int64_t)j * v_stride + c];
        o[c] = (float)acc;
    }
    if (prob_out) for (int32_t j = 0; j < n; ++j) prob_out[j] = (float)p[j];
    free(p);
}

float orc_nll_row(const float *hf, const float *w_lm, int32_t d, int32_t vocab, int32_t target)
{
    float *logit = (float *)malloc(sizeof(float) * (size_t)vocab);
    for (int32_t v = 0; v < vocab; ++v) logit[v] = (float)dot64(w_lm + (int64_t)v * d, hf, d);
    double mx = -INFINITY;
    for (int32_t v = 0; v < vocab; ++v) if ((double)logit[v] > mx) mx = (double)logit[v];
    double se = 0.0;
    for (int32_t v = 0; v < vocab; ++v) se += exp((double)logit[v] - mx);
    double nll = (mx + log(se)) - (double)logit[target];
    free(logit);
    return (float)nll;
}

/* rotary embedding, rotate-half pairing (c, c + head_dim/2), angle pos * theta^(-2c/head_dim) */
static void rope_head(float *x, int32_t head_dim, int32_t pos, float theta)
{
    const int32_t half = head_dim / 2;
    for (int32_t c = 0; c < half; ++c) {
        const double inv_freq = pow((double)theta, -2.0 * (double)c / (double)head_dim);
        const double ang = (double)pos * inv_freq;
        const double cs = cos(ang), sn = sin(ang);
        const double x0 = (double)x[c], x1 = (double)x[c + half];
        x[c]        = (float)(x0 * cs - x1 * sn);
        x[c + half] = (float)(x1 * cs + x0 * sn);
    }
}

/* ------------------------------------------------------------------------ */
/* one decoder layer                                                          */
/* ------------------------------------------------------------------------ */

static int32_t check_cfg(const orc_cfg *cfg, const orc_action *table, int32_t n_actions)
{
    if (!cfg || !table || n_actions <= 0) return -1;
    if (cfg->d_model <= 0 || cfg->n_q_heads <= 0 || cfg->n_kv_heads <= 0 || cfg->head_dim <= 0 ||
        cfg->d_ff <= 0 || (cfg->head_dim & 1) || cfg->n_q_heads % cfg->n_kv_heads != 0 ||
        cfg->page_size < 1 || cfg->n_sink < 0 || cfg->n_window < 0) return -1;
    for (int32_t a = 0; a < n_actions; ++a) {
        const orc_action *t = &table[a];
        if (t->keep_den == 0 || t->keep_num == 0 || t->keep_num > t->keep_den) return -4;
        if (t->mlp_keep_den == 0 || t->mlp_keep_num == 0 || t->mlp_keep_num > t->mlp_keep_den) return -4;
        if (t->bits < 4) return -4;
    }
    return 0;
}

int32_t orc_layer_forward(const orc_cfg *cfg, const orc_action *table, int32_t n_actions,
                          const orc_layer_weights *w,
                          const float *x_in, float *x_out,
                          const int32_t *action_ids, const int32_t *pos0,
                          float *k_cache, float *v_cache,
                          int32_t n_seq, int32_t T, int32_t L_max,
                          const orc_taps *taps)
{
    int32_t rc = check_cfg(cfg, table, n_actions);
    if (rc) return rc;
    if (!w || !x_in || !x_out || !action_ids || !k_cache || !v_cache || n_seq < 0 || T < 0 || L_max <= 0)
        return -1;
    const int32_t d = cfg->d_model, Hq = cfg->n_q_heads, Hkv = cfg->n_kv_heads, dh = cfg->head_dim;
    const int32_t dff = cfg->d_ff, grp = Hq / Hkv, bf = cfg->act_bf16;
    const int64_t M = (int64_t)n_seq * T;
    for (int64_t r = 0; r < M; ++r)
        if (action_ids[r] < 0 || action_ids[r] >= n_actions) return -4;
    for (int32_t s = 0; s < n_seq; ++s) {
        const int32_t p0 = pos0 ? pos0[s] : 0;
        if (p0 < 0 || p0 + T > L_max) return -5;
    }
    if (M == 0) return 0;

    float *h1 = (float *)malloc(sizeof(float) * (size_t)(M * d));
    float *qb = (float *)malloc(sizeof(float) * (size_t)(M * Hq * dh));
    float *ob = (float *)malloc(sizeof(float) * (size_t)(M * Hq * dh));
    float *x2 = (float *)malloc(sizeof(float) * (size_t)(M * d));
    float *h2 = (float *)malloc(sizeof(float) * (size_t)(M * d));
    float *ab = (float *)malloc(sizeof(float) * (size_t)(M * dff));
    const double inv_sqrt_dh = 1.0 / sqrt((double)dh);

    /* steps 1-3: input norm, site A, q/k/v projections, rotary, cache write */
    #pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < M; ++r) {
        const int32_t s = (int32_t)(r / T), i = (int32_t)(r % T);
        const int32_t pos = (pos0 ? pos0[s] : 0) + i;
        const orc_action *act = &table[action_ids[r]];
        float *h = h1 + r * d;
        orc_rmsnorm(x_in + r * d, w->w_in_norm, d, cfg->rms_eps, h);
        if (cfg->quant_sites & ORC_QS_QKV_IN) orc_fake_quant(h, d, (int32_t)act->bits, h, NULL, NULL);
        round_row(h, d, bf);
        float *q = qb + r * Hq * dh;
        matvec(w->wq, h, Hq * dh, d, q);
        for (int32_t hh = 0; hh < Hq; ++hh) rope_head(q + hh * dh, dh, pos, cfg->rope_theta);
        round_row(q, Hq * dh, bf);
        for (int32_t kh = 0; kh < Hkv; ++kh) {
            float *kdst = k_cache + (((int64_t)s * Hkv + kh) * L_max + pos) * dh;
            float *vdst = v_cache + (((int64_t)s * Hkv + kh) * L_max + pos) * dh;
            matvec(w->wk + (int64_t)kh * dh * d, h, dh, d, kdst);
            rope_head(kdst, dh, pos, cfg->rope_theta);
            round_row(kdst, dh, bf);
            matvec(w->wv + (int64_t)kh * dh * d, h, dh, d, vdst);
            round_row(vdst, dh, bf);
        }
    }

    /* steps 4-6: causal scores, budgeted key selection, softmax over kept keys, times V */
    #pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int64_t r = 0; r < M; ++r) {
        for (int32_t hh = 0; hh < Hq; ++hh) {
            const int32_t s = (int32_t)(r / T), i = (int32_t)(r % T);
            const int32_t pos = (pos0 ? pos0[s] : 0) + i;
            const int32_t n = pos + 1;                       /* keys 0..pos, self included */
            const orc_action *act = &table[action_ids[r]];
            const int32_t kh = hh / grp;
            const float *q = qb + (r * Hq + hh) * dh;
            const float *kc = k_cache + ((int64_t)s * Hkv + kh) * L_max * dh;
            const float *vc = v_cache + ((int64_t)s * Hkv + kh) * L_max * dh;
            float *score = (float *)malloc(sizeof(float) * (size_t)n);
            uint8_t *keep = (uint8_t *)malloc((size_t)n);
            for (int32_t j = 0; j < n; ++j)
                score[j] = (float)(dot64(q, kc + (int64_t)j * dh, dh) * inv_sqrt_dh);
            const int32_t b = orc_budget(act->keep_num, act->keep_den, n);
            if (b >= n) {
                memset(keep, 1, (size_t)n);                  /* budget keeps all: dense */
            } else if (cfg->page_size == 1) {
                orc_select_keys(score, n, b, cfg->n_sink, cfg->n_window, keep);
            } else {
                orc_select_pages(q, kc, dh, dh, n, b, cfg->page_size, cfg->n_sink, cfg->n_window, keep, NULL);
            }
            orc_softmax_v(score, keep, n, vc, dh, dh, ob + (r * Hq + hh) * dh, NULL);
            if (taps && taps->keep_mask) {
                uint8_t *dst = taps->keep_mask + ((r * Hq) + hh) * (int64_t)L_max;
                memset(dst, 0, (size_t)L_max);
                memcpy(dst, keep, (size_t)n);
            }
            free(score);
            free(keep);
        }
    }
    if (taps && taps->attn_out) memcpy(taps->attn_out, ob, sizeof(float) * (size_t)(M * Hq * dh));
    if (taps && taps->q_rot) memcpy(taps->q_rot, qb, sizeof(float) * (size_t)(M * Hq * dh));
    if (taps && taps->h1) memcpy(taps->h1, h1, sizeof(float) * (size_t)(M * d));

    /* steps 7-12: site B, output projection + residual, post norm, MLP under prune / quant */
    #pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < M; ++r) {
        const orc_action *act = &table[action_ids[r]];
        const int32_t bits = (int32_t)act->bits;
        float *o = ob + r * Hq * dh;
        if (cfg->quant_sites & ORC_QS_O_IN) orc_fake_quant(o, Hq * dh, bits, o, NULL, NULL);
        round_row(o, Hq * dh, bf);
        float *xm = x2 + r * d;
        matvec(w->wo, o, d, Hq * dh, xm);
        for (int32_t j = 0; j < d; ++j) xm[j] = x_in[r * d + j] + xm[j];

        float *h = h2 + r * d;
        orc_rmsnorm(xm, w->w_post_norm, d, cfg->rms_eps, h);
        if (cfg->prune_site == 1) {
            const int32_t m = orc_budget(act->mlp_keep_num, act->mlp_keep_den, d);
            if (m < d) {
                uint8_t *keep = (uint8_t *)malloc((size_t)d);
                orc_topm_mask(h, d, m, keep);
                for (int32_t j = 0; j < d; ++j) if (!keep[j]) h[j] = 0.0f;
                free(keep);
            }
        }
        if (cfg->quant_sites & ORC_QS_GATEUP_IN) orc_fake_quant(h, d, bits, h, NULL, NULL);
        round_row(h, d, bf);

        float *a = ab + r * dff;
        for (int32_t c = 0; c < dff; ++c) {
            const float gt = (float)dot64(w->w_gate + (int64_t)c * d, h, d);
            const float up = (float)dot64(w->w_up + (int64_t)c * d, h, d);
            const double sg = 1.0 / (1.0 + exp(-(double)gt));
            a[c] = (float)((double)gt * sg * (double)up);
        }
        round_row(a, dff, bf);
        if (cfg->prune_site == 0) {
            const int32_t m = orc_budget(act->mlp_keep_num, act->mlp_keep_den, dff);
            if (m < dff) {
                uint8_t *keep = (uint8_t *)malloc((size_t)dff);
                orc_topm_mask(a, dff, m, keep);
                for (int32_t c = 0; c < dff; ++c) if (!keep[c]) a[c] = 0.0f;
                free(keep);
            }
        }
        if (cfg->quant_sites & ORC_QS_DOWN_IN) orc_fake_quant(a, dff, bits, a, NULL, NULL);
        round_row(a, dff, bf);

        float *z = (float *)malloc(sizeof(float) * (size_t)d);
        matvec(w->w_down, a, d, dff, z);
        if (cfg->quant_sites & ORC_QS_MLP_OUT) orc_fake_quant(z, d, bits, z, NULL, NULL);
        for (int32_t j = 0; j < d; ++j) x_out[r * d + j] = xm[j] + z[j];
        round_row(x_out + r * d, d, bf);
        free(z);
    }
    if (taps && taps->mlp_act) memcpy(taps->mlp_act, ab, sizeof(float) * (size_t)(M * dff));
    if (taps && taps->x_mid) memcpy(taps->x_mid, x2, sizeof(float) * (size_t)(M * d));
    if (taps && taps->h2) memcpy(taps->h2, h2, sizeof(float) * (size_t)(M * d));

    free(h1); free(qb); free(ob); free(x2); free(h2); free(ab);
    return 0;
}

/* ------------------------------------------------------------------------ */
/* decode step: the same layer, one token per sequence, all layers            */
/* ------------------------------------------------------------------------ */
int32_t orc_decode_step(const orc_cfg *cfg, const orc_action *table, int32_t n_actions,
                        const orc_layer_weights *layers,
                        const float *w_final_norm, const float *lm_head,
                        const float *x0, const int32_t *action_ids,
                        const int32_t *cache_len,
                        float *const *k_cache, float *const *v_cache,
                        int32_t B, int32_t L_max,
                        float *hidden_out, const int32_t *targets, float *nll_out)
{
    int32_t rc = check_cfg(cfg, table, n_actions);
    if (rc) return rc;
    if (!layers || !x0 || !action_ids || !cache_len || !k_cache || !v_cache || B < 0) return -1;
    if (nll_out && (!targets || !w_final_norm || !lm_head)) return -1;
    if (B == 0) return 0;
    const int32_t d = cfg->d_model;
    float *xa = (float *)malloc(sizeof(float) * (size_t)B * d);
    float *xb = (float *)malloc(sizeof(float) * (size_t)B * d);
    memcpy(xa, x0, sizeof(float) * (size_t)B * d);
    for (int32_t l = 0; l < cfg->n_layers; ++l) {
        rc = orc_layer_forward(cfg, table, n_actions, &layers[l], xa, xb, action_ids, cache_len,
                               k_cache[l], v_cache[l], B, 1, L_max, NULL);
        if (rc) { free(xa); free(xb); return rc; }
        float *t = xa; xa = xb; xb = t;
    }
    if (hidden_out) memcpy(hidden_out, xa, sizeof(float) * (size_t)B * d);
    if (nll_out) {
        #pragma omp parallel for schedule(dynamic, 1)
        for (int32_t s = 0; s < B; ++s) {
            float *hf = (float *)malloc(sizeof(float) * (size_t)d);
            orc_rmsnorm(xa + (int64_t)s * d, w_final_norm, d, cfg->rms_eps, hf);
            round_row(hf, d, cfg->act_bf16);
            nll_out[s] = orc_nll_row(hf, lm_head, d, cfg->vocab, targets[s]);
            free(hf);
        }
    }
    free(xa); free(xb);
    return 0;
}

/* ------------------------------------------------------------------------ */
/* teacher-forced pass over G compute schedules of the same token path        */
/* ------------------------------------------------------------------------ */
int32_t orc_schedule_loglik(const orc_cfg *cfg, const orc_action *table, int32_t n_actions,
                            const float *embed, const orc_layer_weights *layers,
                            const float *w_final_norm, const float *lm_head,
                            const int32_t *tokens, const int32_t *targets,
                            const int32_t *action_ids,
                            int32_t B, int32_t G, int32_t T,
                            float *nll_out, float *hidden_out)
{
    int32_t rc = check_cfg(cfg, table, n_actions);
    if (rc) return rc;
    if (!embed || !layers || !w_final_norm || !lm_head || !tokens || !targets || !action_ids || !nll_out)
        return -1;
    if (B < 0 || G < 0 || T < 0) return -1;
    const int32_t d = cfg->d_model, N = B * G;
    const int64_t M = (int64_t)N * T;
    if (M == 0) return 0;
    for (int64_t i = 0; i < (int64_t)B * T; ++i) {
        if (tokens[i] < 0 || tokens[i] >= cfg->vocab) return -1;
        if (targets[i] < 0 || targets[i] >= cfg->vocab) return -1;
    }
    float *xa = (float *)malloc(sizeof(float) * (size_t)(M * d));
    float *xb = (float *)malloc(sizeof(float) * (size_t)(M * d));
    const size_t cache_elems = (size_t)N * cfg->n_kv_heads * (size_t)T * cfg->head_dim;
    float *kc = (float *)malloc(sizeof(float) * cache_elems);
    float *vc = (float *)malloc(sizeof(float) * cache_elems);
    /* every schedule g of input b starts from the same embedded tokens */
    for (int32_t b = 0; b < B; ++b)
        for (int32_t g = 0; g < G; ++g)
            for (int32_t t = 0; t < T; ++t)
                memcpy(xa + (((int64_t)b * G + g) * T + t) * d,
                       embed + (int64_t)tokens[(int64_t)b * T + t] * d, sizeof(float) * (size_t)d);
    for (int32_t l = 0; l < cfg->n_layers; ++l) {
        rc = orc_layer_forward(cfg, table, n_actions, &layers[l], xa, xb, action_ids, NULL,
                               kc, vc, N, T, T, NULL);
        if (rc) break;
        float *t = xa; xa = xb; xb = t;
    }
    if (!rc) {
        if (hidden_out) memcpy(hidden_out, xa, sizeof(float) * (size_t)(M * d));
        #pragma omp parallel for schedule(dynamic, 1)
        for (int64_t r = 0; r < M; ++r) {
            const int32_t b = (int32_t)(r / ((int64_t)G * T)), t = (int32_t)(r % T);
            float *hf = (float *)malloc(sizeof(float) * (size_t)d);
            orc_rmsnorm(xa + r * d, w_final_norm, d, cfg->rms_eps, hf);
            round_row(hf, d, cfg->act_bf16);
            nll_out[r] = orc_nll_row(hf, lm_head, d, cfg->vocab, targets[(int64_t)b * T + t]);
            free(hf);
        }
    }
    free(xa); free(xb); free(kc); free(vc);
    return rc;
}
