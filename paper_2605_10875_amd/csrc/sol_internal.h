// Host-visible launchers of the gfx950 kernels. Every launcher only enqueues work on `stream`.
// T-typed pointers are passed as void* with a dtype tag (0 = fp32, 1 = bf16).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "sol_common.h"

namespace sol {

struct ActionDev {  // device copy of one action-table row, with the MLP bucket it belongs to
    uint32_t keep_num, keep_den, mlp_keep_num, mlp_keep_den, bits;
    int32_t  bucket;
};

// ---- rows (sol_rows.hip) ---------------------------------------------------------------------
// Decodes action ids into RowAct (invalid id => dense action + FLAG_BAD_ACTION) and writes each
// row's MLP bucket. d_ff is the width of the vector the MLP keep fraction applies to (d_ff at the
// SiLU(gate)*up site, d_model at the MLP-input site).
void launch_prepare_rows(const int32_t *action_ids, const ActionDev *table, int n_actions, int d_ff,
                         int64_t M, RowAct *ra, int32_t *row_bucket, int *flags, hipStream_t st);
// dst [N][Hkv][L_dst][dh] <- src [N / K][Hkv][P][dh] for positions < P (dh * esize a multiple of 16 bytes).
void launch_bcast_prefix(const void *src, void *dst, int64_t N, int K, int Hkv, int P, int L_dst, int dh, size_t esize,
                         hipStream_t st);
void launch_fill_i32(int32_t *p, int v, int64_t n, hipStream_t st);
// Every row under the dense action (all keys, all `width` channels, no quantiser).
void launch_dense_rows(int width, int64_t M, RowAct *ra, int32_t *row_bucket, hipStream_t st);
// Stable counting sort of rows by bucket: perm[slot] = row, bucket_off[b] = first slot of bucket b
// (n_buckets + 1 entries).
void launch_bucket_sort(const int32_t *row_bucket, int64_t M, int n_buckets, int32_t *perm,
                        int32_t *bucket_off, hipStream_t st);
// h = FQ(RMSNorm(x [+ add]) * w, bits) ; optionally writes xsum = x + add (fp32).
// x: [M][d] of x_dtype; add: fp32 [M][d] or NULL; ra NULL or quant disabled => no quantiser.
// prune: between the norm and the quantiser keep the ra.m largest magnitudes of the row (pruning at the MLP
// input); only the one-wave-per-row kernel does it: false (nothing launched) when that kernel does not cover the
// types / width, and the caller then prunes with launch_prune_fq on an fp32 copy.
bool launch_rmsnorm_fq(const void *x, int x_dtype, const float *add, float *xsum, const void *w, int w_dtype,
                       void *h, int h_dtype, const RowAct *ra, bool quant, int64_t M, int d, float eps,
                       hipStream_t st, int nsplit = 1, bool prune = false);
// out = FQ(in, bits) row-wise; in fp32 [M][n] -> out dtype.
void launch_fq_rows(const float *in, void *out, int out_dtype, const RowAct *ra, bool quant, int64_t M, int n,
                    hipStream_t st);
// rotary + scatter: qkv32 [M][(Hq+2Hkv)*dh] -> q [M][Hq*dh], K/V caches at position pos0[s]+i.
void launch_rope_store(const float *qkv32, void *q, void *k_cache, void *v_cache, int dtype, const float2 *rope,
                       const int32_t *pos0, int n_seq, int T, int L_max, int Hq, int Hkv, int dh, int *flags,
                       hipStream_t st, int nsplit = 1, int cache_rows = 0);
// a = silu(g) * u ; gu32 [M][2*dff] (gate cols first) -> a [M][dff]
void launch_silu_mul(const float *gu32, void *a, int dtype, int64_t M, int dff, hipStream_t st, int nsplit = 1);
// in place on a [M][dff]: keep the ra.m largest |a| (ties to lower channel), then FQ.
// Rows are visited in bucket order through perm (NULL = identity).
// prune = false: no pruning (ra.m then belongs to another site), quantiser only.
void launch_prune_fq(void *a, int dtype, const RowAct *ra, const int32_t *perm, bool quant, int64_t M, int dff,
                     hipStream_t st, bool prune = true);
// whether launch_prune_fq uses perm for this type / width (if not, the bucket sort can be skipped)
bool prune_fq_wants_order(int dtype, int dff);
// out = x2 + z
void launch_resid_out(const float *x2, const float *z, void *out, int dtype, int64_t M, int d, hipStream_t st,
                      int nsplit = 1);
// out = x2 + FQ(z, ra.bits): quantiser on the MLP block's output
void launch_resid_out_fq(const float *x2, const float *z, void *out, int dtype, const RowAct *ra, int64_t M, int d,
                         hipStream_t st, int nsplit = 1);
// x[n][t] = embed[tokens[b][t]]  for n = b*G + g; a token id outside [0, vocab) is clamped and sets FLAG_BAD_TOKEN
// (so do target ids in the two NLL paths below)
void launch_embed(const void *embed, const int32_t *tokens, void *x, int dtype, int B, int G, int T, int d,
                  int vocab, int *flags, hipStream_t st);
// nll[r] = logsumexp(logits[r]) - logits[r][target]; targets indexed through tgt_index(r)
void launch_nll_rows(const float *logits, int64_t rows, int V, const int32_t *targets, int64_t row0, int G, int T,
                     bool broadcast_g, float *nll, int *flags, hipStream_t st);
// unit hooks
// the row stage of the batched threshold kernel on caller rows (n_cols <= 4096, else false and nothing launched)
bool launch_test_attn_threshold(const float *scores, int rows, int n_cols, const int32_t *n_valid, const int32_t *k,
                                uint8_t *keep_out, hipStream_t st);
void launch_test_topk(const float *scores, int rows, int n_cols, const int32_t *n_valid, const int32_t *k,
                      uint8_t *keep, hipStream_t st);
void launch_test_prune(const float *a, int rows, int n, const int32_t *m, uint8_t *keep, hipStream_t st);
// the production prune + quantise kernel on caller rows (scratch: rows * 16 bytes)
void launch_test_prune_quant(void *a, int dtype, int rows, int n, const int32_t *m, const int32_t *bits, void *scratch,
                             hipStream_t st);
void launch_test_quant(const float *z, int rows, int n, const int32_t *bits, int32_t *codes, float *scale,
                       float *zhat, hipStream_t st);

// ---- GEMM (sol_gemm.hip) ---------------------------------------------------------------------
// C[M][N] (fp32, ldc) = A[M][K] (a_dtype, lda) * W[N][K]^T (w_dtype, ldw). Any shape.
void launch_gemm_generic(const void *A, int a_dtype, int64_t lda, const void *W, int w_dtype, int64_t ldw,
                         float *C, int64_t ldc, int64_t M, int N, int K, hipStream_t st);

// ---- bf16 MFMA GEMMs with fused epilogues (sol_gemm_mfma.hip) -----------------------------------
// Each returns false (and launches nothing) if the shape is outside what the tile configuration
// covers; the caller then takes the generic path for that stage.
// q/k/v projections + rotary + q store + K/V cache write.  h: [M][d] bf16. row_sp_ws: 8 bytes per row of
// scratch for the rows' (sequence, position). cache_rows (also of launch_rope_store): rows of one (sequence, KV head)
// in the caches if not L_max; a cache that holds positions [P, P + cache_rows) only is passed as its base minus
// P rows, L_max staying the bound the positions are checked against.
bool launch_gemm_qkv_rope(const void *h, const void *wq, const void *wk, const void *wv, void *q, void *kc, void *vc,
                          const float2 *rope, const int32_t *pos0, int n_seq, int T, int L_max, int Hq, int Hkv, int dh,
                          int d, int *flags, void *row_sp_ws, hipStream_t st, int cache_rows = 0);
// out(fp32)[M][N] = resid(bf16)[M][N] + a[M][K] * w[N][K]^T
bool launch_gemm_resid_f32(const void *a, const void *w, const void *resid, float *out, int64_t M, int N, int K,
                           hipStream_t st);
// a(bf16)[M][dff] = silu(h wg^T) * (h wu^T)
bool launch_gemm_gateup_silu(const void *h, const void *wg, const void *wu, void *a, int64_t M, int dff, int d,
                             hipStream_t st);
// out(bf16)[M][N] = x2(fp32)[M][N] + a[M][K] * w[N][K]^T
bool launch_gemm_resid_out(const void *a, const void *w, const float *x2, void *out, int64_t M, int N, int K,
                           hipStream_t st);
// C(fp32, ldc) = a * w^T
bool launch_gemm_f32(const void *a, const void *w, float *C, int64_t ldc, int64_t M, int N, int K, hipStream_t st);

// LM head + NLL with the logits kept on chip (bf16, vocabulary a multiple of 256): nll[r] = logsumexp - target
// logit. hf must have room for gemm_nll_hf_rows(M) rows (M rounded up to the GEMM's tile; the rows past M are
// cleared by the call); scratch: gemm_nll_scratch_bytes(M, V) bytes.
bool launch_gemm_nll(void *hf, const void *lm_head, const int32_t *targets, int G, int T, bool broadcast_g,
                     float *nll, void *scratch, int64_t M, int V, int K, int *flags, hipStream_t st);
size_t gemm_nll_scratch_bytes(int64_t M, int V);
int64_t gemm_nll_hf_rows(int64_t M);

// Skinny GEMM for M <= 64 rows (decode): partial[nsplit][M][n0+n1+n2] (fp32) = x * [w0; w1; w2]^T, K split over
// nsplit workgroup rows; the consumer kernels above fold the partial sums (their nsplit argument). The fp32
// inputs of those kernels (qkv32 / add / gu32 / z) are then laid out [nsplit][M][N].
bool launch_gemm_skinny(const void *x, int64_t ldx, const void *w0, int n0, const void *w1, int n1, const void *w2,
                        int n2, int M, int K, float *partial, int nsplit, hipStream_t st);
int skinny_splits(int M, int Nv, int K);

// ---- attention (sol_attn.hip) ----------------------------------------------------------------
// One query row per workgroup group: scores over cache positions [0, pos], budgeted top-k,
// softmax over kept keys, times V. o32: fp32 [M][Hq*dh]. Returns false if the shape is unsupported.
// opt: the key-selection rule (page size, sink and window keys); the other attention launchers below
// implement the plain rule only (page 1, no forced keys).
struct AttnOpts {
    int page = 1, n_sink = 0, n_window = 0;
    bool plain() const { return page == 1 && n_sink == 0 && n_window == 0; }
};
bool launch_attn_rows(const void *q, const void *k_cache, const void *v_cache, int dtype, float *o32,
                      const RowAct *ra, const int32_t *pos0, int n_seq, int T, int L_max, int Hq, int Hkv,
                      int dh, int *flags, hipStream_t st, AttnOpts opt = AttnOpts());
// Decode attention: one query per sequence, bf16, 4 query heads per KV head, L_max <= 9216.
void launch_seq_order(const int32_t *cache_len, int B, int32_t *order, hipStream_t st);
bool launch_attn_decode(const void *q, const void *k_cache, const void *v_cache, float *o32, const RowAct *ra,
                        const int32_t *cache_len, const int32_t *seq_order, int B, int L_max, int Hq, int Hkv, int dh,
                        int *flags, hipStream_t st);
// Page metadata of a bf16 K cache for the page rule (page size S >= 2): meta [n_seq][Hkv][ceil(L_max/S)][2*dh],
// per page the channel-wise [maximum | minimum] of its keys. build: from keys [0, len[s]); update: the key at
// pos[s] joins its page. head_dim 64 / 128.
// first (may be NULL): only pages that hold a key >= first[s] are rebuilt; extra: len[s] + extra keys are live.
bool launch_page_meta_build(const void *k_cache, const int32_t *len, void *meta, int n_seq, int L_max, int Hkv, int dh,
                            int S, hipStream_t st, const int32_t *first = nullptr, int extra = 0);
bool launch_page_meta_update(const void *k_cache, const int32_t *pos, void *meta, int n_seq, int L_max, int Hkv, int dh,
                             int S, hipStream_t st);
// Decode attention under the page rule with that metadata (which must already include the new key).
bool launch_attn_decode_paged(const void *q, const void *k_cache, const void *v_cache, const void *meta, float *o32,
                              const RowAct *ra, const int32_t *cache_len, const int32_t *seq_order, int B, int L_max, int Hq,
                              int Hkv, int dh, AttnOpts opt, int *flags, hipStream_t st);
// A prefix cache shared by groups of K consecutive sequences (the schedules of one input): keys [0, P) of sequence s
// come from k / vt of input s / K ([inputs][Hkv][P][dh], transposed copy [inputs][Hkv][dh][lpadv]); the sequence's own
// cache then holds positions P.. only, crows rows per (sequence, KV head). P a multiple of 64.
struct PrefixView {
    const bf16_t *k = nullptr, *vt = nullptr;
    const bf16_t *kf = nullptr;           // optional: the prefix K caches in MFMA operand order (launch_attn_frag_k)
    int P = 0, K = 1, lpadv = 0, crows = 0;
    const bf16_t *pm = nullptr;           // page rule: metadata rows of the prefix keys ([inputs][Hkv][P][2 * dh])
};
bool launch_page_prefix_meta(const void *k_cache, void *pm, int n_seq, int P, int Hkv, int dh, int S, hipStream_t st);
bool attn_tile_pages_prefix_ok(int n_seq, int T, int Hq, int Hkv, int dh, int S, const PrefixView &pv);
bool launch_attn_tile_pages_prefix(const void *q, const void *k_cache, const void *v_cache, void *vt, void *pm, void *selp,
                                   float *o32, const RowAct *ra, const int32_t *pos0, int n_seq, int T, int Hq, int Hkv,
                                   int dh, AttnOpts opt, PrefixView pv, hipStream_t st);
// Batched bf16 attention (L_max <= 4096, head_dim 64 or 128, 1/2/4/8 query heads per KV head): a threshold
// kernel followed by a flash-style masked softmax * V kernel. vt is workspace for the transposed V copy
// (n_seq * Hkv * dh * attn_tile_lpadv(L_max) elements), kfr for the copy of K in MFMA operand order (as many),
// sel_ws for the per-(row, head) thresholds (attn_tile_sel_bytes(rows, Hq) bytes).
bool launch_attn_tile(const void *q, const void *k_cache, const void *v_cache, void *vt, void *kfr, void *sel_ws, float *o32,
                      const RowAct *ra, const int32_t *pos0, int n_seq, int T, int L_max, int Hq, int Hkv, int dh,
                      hipStream_t st);
size_t attn_tile_sel_bytes(int64_t rows, int Hq);
// K cache [n_seq][Hkv][L_max][dh] -> kfr [n_seq][Hkv][attn_tile_lpadv(L_max) / 16][dh / 32][64][8], the order in which
// the threshold kernel's MFMAs take it (keys from pos0[s] + T on are zero; pos0 == nullptr: 0). False: head size.
bool launch_attn_frag_k(const void *k_cache, void *kfr, const int32_t *pos0, int n_seq, int T, int L_max, int Hkv, int dh,
                        hipStream_t st);
// The same for sequences that share prefix caches: k_cache / v_cache hold positions pv.P.. only, vt is scratch for
// their transposed copy (n_seq * Hkv * dh * attn_tile_lpadv(pv.crows) elements); the T rows of every sequence sit at
// positions pv.P.. (pos0 must say so). False if a shape or address limit is not met (nothing launched).
bool attn_tile_prefix_ok(const void *k_cache, int n_seq, int T, int Hq, int Hkv, int dh, const PrefixView &pv);
bool launch_attn_tile_prefix(const void *q, const void *k_cache, const void *v_cache, void *vt, void *sel_ws, float *o32,
                             const RowAct *ra, const int32_t *pos0, int n_seq, int T, int Hq, int Hkv, int dh, PrefixView pv,
                             hipStream_t st);
// The same under the page rule (page size a power of two in [4, 64], at most 256 pages) with sink / window keys:
// per-key prefix extremes of the pages (pm scratch), a bit mask of kept pages per (row, head) (selp scratch), then
// the flash-style kernel with a running maximum.
bool launch_attn_tile_pages(const void *q, const void *k_cache, const void *v_cache, void *vt, void *pm, void *selp,
                            float *o32, const RowAct *ra, const int32_t *pos0, int n_seq, int T, int L_max, int Hq, int Hkv,
                            int dh, AttnOpts opt, hipStream_t st);
size_t attn_tile_pages_meta_bytes(int64_t n_seq, int Hkv, int L_max, int dh);
// Dense causal attention (every row keeps every key): the flash-style kernel alone. Shapes of launch_attn_tile.
bool launch_attn_tile_dense(const void *q, const void *k_cache, const void *v_cache, void *vt, float *o32,
                            const int32_t *pos0, int n_seq, int T, int L_max, int Hq, int Hkv, int dh, hipStream_t st);
size_t attn_tile_pages_sel_bytes(int64_t rows, int Hq, int L_max, int S);
int attn_tile_lpadv(int L_max);

// ---- reward reduction (sol_reward.hip) ----------------------------------------------------------
struct RewardCfg { float alpha_kappa, alpha_rho, alpha_eta, tau, gamma, eps; };
// nll, ids [B][K][T]; eff [B][T] or NULL; targets [B][3]; avg_out [B][K][3], pen_out [B][K], ret_out [B][K][T] may be
// NULL; signal and adv [B][K][T]; scratch: reward_scratch_bytes(B, T).
void launch_reward(const float *nll, const int32_t *ids, const ActionDev *table, int n_actions, const int32_t *eff,
                   const float *targets, const RewardCfg &rc, int B, int K, int T, float *avg_out, float *pen_out,
                   float *ret_out, float *signal, float *adv, void *scratch, int *flags, hipStream_t st);
size_t reward_scratch_bytes(int B, int T);

}  // namespace sol
