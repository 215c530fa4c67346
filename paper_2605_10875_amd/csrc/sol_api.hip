// Host side of the C ABI: validation, context, workspace carve-up and the launch sequence of the
// action-conditioned decoder layer, the decode step and the teacher-forced schedule pass.
#include "../../include/sol.h"

#include <cmath>
#include <cstdio>
#include <cstring>
#include <map>
#include <string>
#include <utility>
#include <vector>

#include "sol_internal.h"

using namespace sol;

enum Stage {
    ST_PREPARE = 0, ST_NORM_IN, ST_QKV, ST_ROPE, ST_ATTN, ST_QUANT_O, ST_OPROJ, ST_NORM_POST, ST_GATEUP, ST_SILU,
    ST_PRUNE, ST_DOWN, ST_RESID, ST_EMBED, ST_NORM_FINAL, ST_LMHEAD, ST_NLL, ST_COUNT
};
static const char *const STAGE_NAMES[ST_COUNT] = {
    "prepare_actions", "norm_in_quant", "qkv_gemm", "rope_cache_write", "attention_topk", "quant_o", "o_proj_gemm",
    "norm_post_quant", "gate_up_gemm", "silu_mul", "prune_quant", "down_gemm", "residual_out", "embed",
    "norm_final", "lm_head_gemm", "nll_rows"};

// Scratch of sol_decode_step_static: callers that cannot allocate get the decode step's workspace from this
// file-scope array instead. Every GPU holds its own copy at its own address; host code must not use the array's name
// as an address but the pointer hipGetSymbolAddress returns for the current device (kept per context below).
#define SOL_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
static __device__ __align__(256) unsigned char scratch[SOL_STATIC_SCRATCH_BYTES];

struct sol_ctx {
    sol_model_cfg cfg;
    int device = -1;               // the HIP device the context was created on
    void *static_scratch = nullptr;    // that device's address of `scratch`
    int n_actions = 0;
    int n_buckets = 1;
    ActionDev *d_table = nullptr;
    float2 *d_rope = nullptr;
    int *d_flags = nullptr;
    std::string err;
    // optional per-stage timing (sol_profile_*): pairs of events recorded around each stage
    bool prof = false;
    std::vector<hipEvent_t> ev;
    std::vector<int> ev_stage;     // stage of pair i (events 2i, 2i+1)
    size_t ev_used = 0;
};

// Brackets one stage with events on the stream while profiling is on (no-op otherwise).
struct StageTimer {
    sol_ctx *c; hipStream_t st; bool on;
    StageTimer(sol_ctx *ctx, int stage, hipStream_t s) : c(ctx), st(s), on(false)
    {
        if (!c->prof || 2 * (c->ev_used + 1) > c->ev.size()) return;
        on = true;
        c->ev_stage[c->ev_used] = stage;
        (void)hipEventRecord(c->ev[2 * c->ev_used], st);
    }
    ~StageTimer()
    {
        if (!on) return;
        (void)hipEventRecord(c->ev[2 * c->ev_used + 1], st);
        c->ev_used++;
    }
};
#define STAGE(ctx, id, st) StageTimer stage_timer_##id(ctx, id, st)

static thread_local std::string g_create_err;
static const int MAX_ACTIONS = 4096;

static int fail(sol_ctx *ctx, int code, const std::string &msg)
{
    if (ctx) ctx->err = msg; else g_create_err = msg;
    return code;
}

#define SOL_HIP(ctx, call)                                                                            \
    do {                                                                                              \
        hipError_t e_ = (call);                                                                       \
        if (e_ != hipSuccess)                                                                         \
            return fail(ctx, SOL_ERR_HIP, std::string(#call) + ": " + hipGetErrorString(e_));         \
    } while (0)

static size_t esize(int dtype) { return dtype == SOL_BF16 ? 2 : 4; }

// ------------------------------------------------------------------------------------------------
// validation (host only)
// ------------------------------------------------------------------------------------------------
static int validate(const sol_model_cfg *c, const sol_action_def *t, int n, std::string &msg)
{
    if (!c) { msg = "cfg is NULL"; return SOL_ERR_INVALID_ARG; }
    if (c->d_model <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0 || c->head_dim <= 0 || c->d_ff <= 0 ||
        c->n_layers <= 0 || c->vocab < 0 || c->max_positions <= 0) {
        msg = "non-positive model dimension"; return SOL_ERR_INVALID_ARG;
    }
    if (c->n_q_heads % c->n_kv_heads) { msg = "n_q_heads must be a multiple of n_kv_heads"; return SOL_ERR_INVALID_ARG; }
    if (c->head_dim & 1) { msg = "head_dim must be even (rotary pairs)"; return SOL_ERR_INVALID_ARG; }
    if (!(c->rms_eps >= 0.f) || !(c->rope_theta > 0.f)) { msg = "bad rms_eps / rope_theta"; return SOL_ERR_INVALID_ARG; }
    if (c->dtype != SOL_F32 && c->dtype != SOL_BF16) { msg = "dtype must be SOL_F32 or SOL_BF16"; return SOL_ERR_INVALID_ARG; }
    if (c->page_size < 1 || c->n_sink < 0 || c->n_window < 0) { msg = "bad page_size / n_sink / n_window"; return SOL_ERR_INVALID_ARG; }
    if (!t || n <= 0) { msg = "empty action table"; return SOL_ERR_INVALID_ARG; }
    if (n > MAX_ACTIONS) { msg = "more than 4096 actions"; return SOL_ERR_UNSUPPORTED; }
    for (int a = 0; a < n; ++a) {
        const sol_action_def &d = t[a];
        if (d.keep_den == 0 || d.keep_num == 0 || d.keep_num > d.keep_den) {
            msg = "action " + std::to_string(a) + ": attention keep fraction must be in (0,1]"; return SOL_ERR_ACTION;
        }
        if (d.mlp_keep_den == 0 || d.mlp_keep_num == 0 || d.mlp_keep_num > d.mlp_keep_den) {
            msg = "action " + std::to_string(a) + ": MLP keep fraction must be in (0,1]"; return SOL_ERR_ACTION;
        }
        if (d.bits < 4) { msg = "action " + std::to_string(a) + ": bits must be >= 4"; return SOL_ERR_ACTION; }
    }
    if (c->prune_site != 0 && c->prune_site != 1) { msg = "prune_site must be 0 or 1"; return SOL_ERR_INVALID_ARG; }
    if (c->quant_sites & ~(SOL_QS_ALL_LINEAR_INPUTS | SOL_QS_MLP_OUT)) { msg = "unknown quant site bit"; return SOL_ERR_INVALID_ARG; }
    const int vec = c->dtype == SOL_BF16 ? 8 : 4;
    const int lpk = c->head_dim / vec;
    if (c->head_dim % vec || lpk > 64 || (lpk & (lpk - 1))) {
        msg = "head_dim must be 8*2^k (bf16) or 4*2^k (fp32), at most 512/256"; return SOL_ERR_UNSUPPORTED;
    }
    return SOL_OK;
}

extern "C" int sol_validate_config(const sol_model_cfg *cfg, const sol_action_def *table, int n_actions)
{
    std::string msg;
    const int rc = validate(cfg, table, n_actions, msg);
    if (rc) g_create_err = msg;
    return rc;
}

extern "C" const char *sol_last_error(const sol_ctx *ctx) { return ctx ? ctx->err.c_str() : g_create_err.c_str(); }

// ------------------------------------------------------------------------------------------------
// context
// ------------------------------------------------------------------------------------------------
extern "C" int sol_create(const sol_model_cfg *cfg, const sol_action_def *table, int n_actions, sol_ctx **out)
{
    if (!out) return fail(nullptr, SOL_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    std::string msg;
    int rc = validate(cfg, table, n_actions, msg);
    if (rc) return fail(nullptr, rc, msg);
    sol_ctx *ctx = new sol_ctx();
    ctx->cfg = *cfg;
    ctx->n_actions = n_actions;
    // MLP buckets: actions that share (kept channels, effective bit-width) share a bucket
    std::vector<ActionDev> host(n_actions);
    std::map<std::pair<int64_t, int>, int> bucket_of;
    const bool q_down = (cfg->quant_sites & SOL_QS_DOWN_IN) != 0;
    for (int a = 0; a < n_actions; ++a) {
        const sol_action_def &d = table[a];
        uint64_t m = ((uint64_t)d.mlp_keep_num * (uint64_t)cfg->d_ff + d.mlp_keep_den - 1) / d.mlp_keep_den;
        if (m < 1) m = 1;
        if (m > (uint64_t)cfg->d_ff) m = (uint64_t)cfg->d_ff;
        const int b_eff = (!q_down || d.bits >= 16) ? 16 : (int)d.bits;
        bucket_of.emplace(std::make_pair(-(int64_t)m, -b_eff), 0);   // dense-most bucket first
    }
    int nb = 0;
    for (auto &kv : bucket_of) kv.second = nb++;
    ctx->n_buckets = nb;
    for (int a = 0; a < n_actions; ++a) {
        const sol_action_def &d = table[a];
        uint64_t m = ((uint64_t)d.mlp_keep_num * (uint64_t)cfg->d_ff + d.mlp_keep_den - 1) / d.mlp_keep_den;
        if (m < 1) m = 1;
        if (m > (uint64_t)cfg->d_ff) m = (uint64_t)cfg->d_ff;
        const int b_eff = (!q_down || d.bits >= 16) ? 16 : (int)d.bits;
        host[a] = ActionDev{d.keep_num, d.keep_den, d.mlp_keep_num, d.mlp_keep_den, d.bits,
                            bucket_of[std::make_pair(-(int64_t)m, -b_eff)]};
    }
    // rotary table: cos/sin(pos * theta^(-2c/dh)), double precision on the host
    const int half = cfg->head_dim / 2;
    std::vector<float2> rope((size_t)cfg->max_positions * half);
    for (int c = 0; c < half; ++c) {
        const double inv_freq = std::pow((double)cfg->rope_theta, -2.0 * (double)c / (double)cfg->head_dim);
        for (int p = 0; p < cfg->max_positions; ++p) {
            const double ang = (double)p * inv_freq;
            rope[(size_t)p * half + c] = make_float2((float)std::cos(ang), (float)std::sin(ang));
        }
    }
    auto cleanup = [&](int code, const std::string &m2) {
        if (ctx->d_table) (void)hipFree(ctx->d_table);
        if (ctx->d_rope) (void)hipFree(ctx->d_rope);
        if (ctx->d_flags) (void)hipFree(ctx->d_flags);
        delete ctx;
        return fail(nullptr, code, m2);
    };
    hipError_t e;
    if ((e = hipGetDevice(&ctx->device)) != hipSuccess)
        return cleanup(SOL_ERR_HIP, std::string("hipGetDevice: ") + hipGetErrorString(e));
    if ((e = hipGetSymbolAddress(&ctx->static_scratch, HIP_SYMBOL(scratch))) != hipSuccess || !ctx->static_scratch)
        return cleanup(SOL_ERR_HIP, std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e));
    if ((e = hipMalloc((void **)&ctx->d_table, sizeof(ActionDev) * n_actions)) != hipSuccess)
        return cleanup(SOL_ERR_HIP, std::string("hipMalloc(table): ") + hipGetErrorString(e));
    if ((e = hipMalloc((void **)&ctx->d_rope, sizeof(float2) * rope.size())) != hipSuccess)
        return cleanup(SOL_ERR_HIP, std::string("hipMalloc(rope): ") + hipGetErrorString(e));
    if ((e = hipMalloc((void **)&ctx->d_flags, 256)) != hipSuccess)
        return cleanup(SOL_ERR_HIP, std::string("hipMalloc(flags): ") + hipGetErrorString(e));
    if ((e = hipMemcpy(ctx->d_table, host.data(), sizeof(ActionDev) * n_actions, hipMemcpyHostToDevice)) != hipSuccess ||
        (e = hipMemcpy(ctx->d_rope, rope.data(), sizeof(float2) * rope.size(), hipMemcpyHostToDevice)) != hipSuccess ||
        (e = hipMemset(ctx->d_flags, 0, 256)) != hipSuccess)
        return cleanup(SOL_ERR_HIP, std::string("upload: ") + hipGetErrorString(e));
    *out = ctx;
    return SOL_OK;
}

extern "C" void sol_destroy(sol_ctx *ctx)
{
    if (!ctx) return;
    (void)hipFree(ctx->d_table);
    (void)hipFree(ctx->d_rope);
    (void)hipFree(ctx->d_flags);
    for (hipEvent_t e : ctx->ev) (void)hipEventDestroy(e);
    delete ctx;
}

extern "C" int sol_profile_enable(sol_ctx *ctx, int max_stage_records)
{
    if (!ctx) return SOL_ERR_INVALID_ARG;
    if (max_stage_records <= 0) { ctx->prof = false; return SOL_OK; }
    while (ctx->ev.size() < 2 * (size_t)max_stage_records) {
        hipEvent_t e;
        SOL_HIP(ctx, hipEventCreate(&e));
        ctx->ev.push_back(e);
    }
    ctx->ev_stage.resize(ctx->ev.size() / 2);
    ctx->ev_used = 0;
    ctx->prof = true;
    return SOL_OK;
}

extern "C" int sol_profile_read(sol_ctx *ctx, void *stream, int max_stages, const char **names_out, float *ms_out,
                                int *calls_out)
{
    if (!ctx || !names_out || !ms_out || !calls_out || max_stages < 0) return SOL_ERR_INVALID_ARG;
    SOL_HIP(ctx, hipStreamSynchronize((hipStream_t)stream));
    const int n = max_stages < (int)ST_COUNT ? max_stages : (int)ST_COUNT;
    for (int i = 0; i < n; ++i) { names_out[i] = STAGE_NAMES[i]; ms_out[i] = 0.f; calls_out[i] = 0; }
    for (size_t i = 0; i < ctx->ev_used; ++i) {
        float ms = 0.f;
        SOL_HIP(ctx, hipEventElapsedTime(&ms, ctx->ev[2 * i], ctx->ev[2 * i + 1]));
        const int sidx = ctx->ev_stage[i];
        if (sidx < n) { ms_out[sidx] += ms; calls_out[sidx] += 1; }
    }
    ctx->ev_used = 0;
    return n;
}

extern "C" int sol_device_status(sol_ctx *ctx, void *stream)
{
    if (!ctx) return SOL_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    SOL_HIP(ctx, hipStreamSynchronize(st));
    int f = 0;
    SOL_HIP(ctx, hipMemcpy(&f, ctx->d_flags, sizeof(int), hipMemcpyDeviceToHost));
    if (f) SOL_HIP(ctx, hipMemset(ctx->d_flags, 0, sizeof(int)));
    if (f & FLAG_CACHE_OVERFLOW) return fail(ctx, SOL_ERR_CACHE_OVERFLOW, "a sequence's tokens did not fit its cache and were skipped");
    if (f & FLAG_BAD_ACTION) return fail(ctx, SOL_ERR_ACTION, "an action id outside the table was treated as the dense action");
    if (f & FLAG_BAD_TOKEN) return fail(ctx, SOL_ERR_INVALID_ARG, "a token or target id outside the vocabulary was clamped into it");
    return SOL_OK;
}

// ------------------------------------------------------------------------------------------------
// workspace
// ------------------------------------------------------------------------------------------------
struct Carver {
    char *base;
    size_t off = 0;
    explicit Carver(void *b) : base((char *)b) {}
    void *take(size_t bytes)
    {
        off = (off + 255) & ~(size_t)255;
        void *p = base ? base + off : nullptr;
        off += bytes;
        return p;
    }
};

struct LayerWs {
    RowAct *ra; int32_t *row_bucket, *perm, *bucket_off, *seq_order;
    void *h, *qb, *a, *vt, *kf, *pm;
    float *big32, *o32, *x2, *hn32;
};

static void carve_layer(Carver &c, const sol_model_cfg &g, int64_t n_seq, int64_t T, int L_max, LayerWs &w)
{
    const int64_t M = n_seq * T;
    const size_t es = esize(g.dtype);
    const int64_t nq = (int64_t)g.n_q_heads * g.head_dim, nkv = (int64_t)g.n_kv_heads * g.head_dim;
    int64_t wide = nq + 2 * nkv;
    if (2 * (int64_t)g.d_ff > wide) wide = 2 * (int64_t)g.d_ff;
    if (g.d_model > wide) wide = g.d_model;
    w.ra = (RowAct *)c.take(sizeof(RowAct) * M);
    w.row_bucket = (int32_t *)c.take(4 * M);
    w.perm = (int32_t *)c.take(4 * M);
    w.bucket_off = (int32_t *)c.take(4 * (MAX_ACTIONS + 1));
    w.seq_order = (int32_t *)c.take(4 * n_seq);
    w.h = c.take(es * M * g.d_model);
    w.qb = c.take(es * M * nq);
    w.a = c.take(es * M * g.d_ff);
    if (g.dtype == SOL_BF16 && M <= 64) {               // decode: K-split partial sums of the skinny GEMMs
        const int64_t cand[4] = {(int64_t)skinny_splits((int)M, (int)(nq + 2 * nkv), g.d_model) * (nq + 2 * nkv),
                                 (int64_t)skinny_splits((int)M, g.d_model, (int)nq) * g.d_model,
                                 (int64_t)skinny_splits((int)M, 2 * g.d_ff, g.d_model) * 2 * g.d_ff,
                                 (int64_t)skinny_splits((int)M, g.d_model, g.d_ff) * g.d_model};
        for (int64_t v : cand) if (v > wide) wide = v;
    }
    w.big32 = (float *)c.take(4 * M * wide);
    w.o32 = (float *)c.take(4 * M * nq);
    w.x2 = (float *)c.take(4 * M * g.d_model);
    w.hn32 = (float *)c.take(g.prune_site == 1 ? 4 * M * g.d_model : 0);   // fp32 post-norm row, pruned at the MLP input
    // transposed V copy for the tiled attention kernel (batched bf16 pass only)
    const bool tiled = g.dtype == SOL_BF16 && T >= 16 && L_max <= 4096;
    w.vt = c.take(tiled ? es * n_seq * g.n_kv_heads * g.head_dim * (size_t)attn_tile_lpadv(L_max) : 0);
    // K in MFMA operand order for the threshold kernel
    w.kf = c.take(tiled ? es * n_seq * g.n_kv_heads * g.head_dim * (size_t)attn_tile_lpadv(L_max) : 0);
    // per-key page extremes for the tiled kernels under the page rule
    w.pm = c.take(tiled && g.page_size > 1 ? attn_tile_pages_meta_bytes(n_seq, g.n_kv_heads, L_max, g.head_dim) : 0);
}

static int64_t lm_chunk_rows(const sol_model_cfg &g, int64_t M)
{
    int64_t rows = (int64_t)(256u << 20) / (4 * (int64_t)(g.vocab > 0 ? g.vocab : 1));
    if (rows < 64) rows = 64;
    return rows < M ? rows : M;
}

struct StackWs {
    LayerWs layer;
    void *xa, *xb, *hf, *kc, *vc;
    float *logits;
};

static void carve_stack(Carver &c, const sol_model_cfg &g, int64_t n_seq, int64_t T, bool own_cache, StackWs &w)
{
    const size_t es = esize(g.dtype);
    const int64_t M = n_seq * T;
    carve_layer(c, g, n_seq, T, own_cache ? (int)T : 1 << 30, w.layer);
    w.xa = c.take(es * M * g.d_model);
    w.xb = c.take(es * M * g.d_model);
    w.hf = c.take(es * gemm_nll_hf_rows(M) * g.d_model);          // the fused LM head reads whole tiles of rows
    const size_t cache = own_cache ? es * n_seq * g.n_kv_heads * T * g.head_dim : 0;
    w.kc = c.take(cache);
    w.vc = c.take(cache);
    size_t head_bytes = 4 * lm_chunk_rows(g, M) * (size_t)(g.vocab > 0 ? g.vocab : 1);          // a chunk of logits rows
    if (g.dtype == SOL_BF16 && g.vocab > 0 && g.vocab % 256 == 0 && gemm_nll_scratch_bytes(M, g.vocab) > head_bytes)
        head_bytes = gemm_nll_scratch_bytes(M, g.vocab);                                         // fused LM head + NLL
    w.logits = (float *)c.take(head_bytes);
}

extern "C" size_t sol_workspace_bytes(const sol_model_cfg *cfg, int op, int n_seq, int T, int L_max)
{
    (void)L_max;
    if (!cfg || n_seq <= 0) return 0;
    Carver c(nullptr);
    if (op == SOL_OP_LAYER_FORWARD) {
        if (T <= 0) return 0;
        LayerWs w; carve_layer(c, *cfg, n_seq, T, L_max, w);
    } else if (op == SOL_OP_DECODE_STEP) {
        StackWs w; carve_stack(c, *cfg, n_seq, 1, false, w);
    } else if (op == SOL_OP_SCHEDULE_LOGLIK) {
        if (T <= 0) return 0;
        StackWs w; carve_stack(c, *cfg, n_seq, T, true, w);
    } else if (op == SOL_OP_REWARD) {
        if (T <= 0) return 0;
        return reward_scratch_bytes(n_seq, T) + 256;
    } else if (op == SOL_OP_KV_REFRESH) {
        if (T <= 0 || L_max <= 0) return 0;
        LayerWs w; carve_layer(c, *cfg, n_seq, T, L_max, w);
        const size_t es = esize(cfg->dtype);
        c.take(es * (size_t)n_seq * T * cfg->d_model);
        c.take(es * (size_t)n_seq * T * cfg->d_model);
    } else return 0;
    return c.off + 256;
}

// ------------------------------------------------------------------------------------------------
// the layer
// ------------------------------------------------------------------------------------------------
static void prepare_actions(sol_ctx *ctx, const int32_t *ids, int64_t M, LayerWs &w, hipStream_t st)
{
    STAGE(ctx, ST_PREPARE, st);
    launch_prepare_rows(ids, ctx->d_table, ctx->n_actions, ctx->cfg.prune_site ? ctx->cfg.d_model : ctx->cfg.d_ff, M,
                        w.ra, w.row_bucket, ctx->d_flags, st);
    if (prune_fq_wants_order(ctx->cfg.dtype, ctx->cfg.d_ff))
        launch_bucket_sort(w.row_bucket, M, ctx->n_buckets, w.perm, w.bucket_off, st);
}

// Few rows (a decode step): the linear layers are bound by reading their weights once and take the skinny GEMM.
static bool use_skinny(const sol_model_cfg &g, int64_t M)
{
    return g.dtype == SOL_BF16 && M <= 64 && g.d_model % 64 == 0 && (g.n_q_heads * g.head_dim) % 64 == 0 && g.d_ff % 64 == 0;
}

// Attention stage of the layer: causal scores over cache positions [0, pos], the budgeted selection of the token's
// action, softmax over the kept keys, times V. Reads w.qb and the caches, writes w.o32 (fp32, before the quantiser of
// the output projection's input); w.vt / w.pm / w.big32 are scratch.
static int attn_stage(sol_ctx *ctx, LayerWs &w, const int32_t *pos0, void *kc, void *vc, int n_seq, int T, int L_max,
                      hipStream_t st, void *page_meta, bool dense_pass, const PrefixView *pv)
{
    const sol_model_cfg &g = ctx->cfg;
    const int dt = g.dtype;
    const int64_t M = (int64_t)n_seq * T;
    const int Hq = g.n_q_heads, Hkv = g.n_kv_heads, dh = g.head_dim;
    const int nqkv = (Hq + 2 * Hkv) * dh;
    const bool mfma = dt == SOL_BF16;
    {
        STAGE(ctx, ST_ATTN, st);
        AttnOpts opt;
        if (!dense_pass) { opt.page = g.page_size; opt.n_sink = g.n_sink; opt.n_window = g.n_window; }   // dense rows keep every key under any rule
        const bool fast = mfma && opt.plain();       // the tiled and decode kernels know the plain top-k rule only
        if (pv) {   // sequences on shared prefix caches: the tiled kernels with two-segment addressing, or nothing
            bool ok = mfma && w.vt;
            if (ok && opt.plain())
                ok = launch_attn_tile_prefix(w.qb, kc, vc, w.vt, w.big32, w.o32, w.ra, pos0, n_seq, T, Hq, Hkv, dh, *pv, st);
            else if (ok)   // page rule (the masks live in big32)
                ok = opt.page > 1 && w.pm && attn_tile_pages_sel_bytes(M, Hq, pv->P + T, opt.page) <= 4 * (size_t)M * nqkv &&
                     launch_attn_tile_pages_prefix(w.qb, kc, vc, w.vt, w.pm, w.big32, w.o32, w.ra, pos0, n_seq, T, Hq, Hkv,
                                                   dh, opt, *pv, st);
            if (!ok) return fail(ctx, SOL_ERR_UNSUPPORTED, "shared-prefix attention: shape outside the tiled kernels");
        }
        bool tiled = pv != nullptr;
        tiled = tiled || (dense_pass && mfma && w.vt && T >= 16 && L_max <= 4096 &&
                          launch_attn_tile_dense(w.qb, kc, vc, w.vt, w.o32, pos0, n_seq, T, L_max, Hq, Hkv, dh, st));
        tiled = tiled || (fast && w.vt && w.kf && T >= 16 && L_max <= 4096 &&
                          launch_attn_tile(w.qb, kc, vc, w.vt, w.kf, w.big32, w.o32, w.ra, pos0, n_seq, T, L_max, Hq, Hkv, dh, st));
        if (!tiled && mfma && opt.page > 1 && w.vt && w.pm && T >= 16 && L_max <= 4096 &&
            attn_tile_pages_sel_bytes(M, Hq, L_max, opt.page) <= 4 * (size_t)M * nqkv)   // the masks live in big32
            tiled = launch_attn_tile_pages(w.qb, kc, vc, w.vt, w.pm, w.big32, w.o32, w.ra, pos0, n_seq, T, L_max, Hq, Hkv, dh, opt, st);
        bool dec = !tiled && fast && T == 1 && pos0 &&
                   launch_attn_decode(w.qb, kc, vc, w.o32, w.ra, pos0, w.seq_order, n_seq, L_max, Hq, Hkv, dh, ctx->d_flags, st);
        if (!tiled && !dec && mfma && T == 1 && pos0 && page_meta && opt.page > 1) {
            // page rule with caller-kept metadata: the new key joins its page, then bounds come from the metadata
            dec = launch_page_meta_update(kc, pos0, page_meta, n_seq, L_max, Hkv, dh, opt.page, st) &&
                  launch_attn_decode_paged(w.qb, kc, vc, page_meta, w.o32, w.ra, pos0, w.seq_order, n_seq, L_max, Hq, Hkv,
                                           dh, opt, ctx->d_flags, st);
            if (!dec) return fail(ctx, SOL_ERR_UNSUPPORTED, "paged decode attention: more pages or keys than the kernel holds on chip");
        }
        if (!tiled && !dec &&
            !launch_attn_rows(w.qb, kc, vc, dt, w.o32, w.ra, pos0, n_seq, T, L_max, Hq, Hkv, dh, ctx->d_flags, st, opt))
            return fail(ctx, SOL_ERR_UNSUPPORTED, "attention: L_max too long for the on-chip score rows of this build");
    }
    return SOL_OK;
}

// MLP stage of the layer from its input on: gate / up projections, SiLU(gate)*up, magnitude pruning and the
// quantiser of the down projection's input, down projection, (quantiser of the MLP output,) residual add.
// Reads w.h (the MLP input as the projections take it) and w.x2 (fp32 residual after attention), writes w.a and x_out.
static int mlp_stage(sol_ctx *ctx, const sol_layer_weights *lw, LayerWs &w, void *x_out, int64_t M, bool skinny,
                     hipStream_t st)
{
    const sol_model_cfg &g = ctx->cfg;
    const int dt = g.dtype;
    const int d = g.d_model, dff = g.d_ff;
    const uint32_t qs = g.quant_sites;
    const bool mfma = dt == SOL_BF16;
    bool fused_gu = false;
    int ns_gu = 1;
    {   // gate / up (+ SiLU(gate)*up when fused)
        STAGE(ctx, ST_GATEUP, st);
        if (skinny) {
            ns_gu = skinny_splits((int)M, 2 * dff, d);
            if (!launch_gemm_skinny(w.h, d, lw->w_gate, dff, lw->w_up, dff, nullptr, 0, (int)M, d, w.big32, ns_gu, st))
                return fail(ctx, SOL_ERR_UNSUPPORTED, "skinny GEMM (gate / up): unsupported shape");
        } else {
            fused_gu = mfma && launch_gemm_gateup_silu(w.h, lw->w_gate, lw->w_up, w.a, M, dff, d, st);
            if (!fused_gu) {
                launch_gemm_generic(w.h, dt, d, lw->w_gate, dt, d, w.big32, 2 * (int64_t)dff, M, dff, d, st);
                launch_gemm_generic(w.h, dt, d, lw->w_up, dt, d, w.big32 + dff, 2 * (int64_t)dff, M, dff, d, st);
            }
        }
    }
    if (!fused_gu) {   // SiLU(gate)*up
        STAGE(ctx, ST_SILU, st);
        launch_silu_mul(w.big32, w.a, dt, M, dff, st, ns_gu);
    }
    {   // magnitude pruning + quantise (down input), rows visited in bucket order
        STAGE(ctx, ST_PRUNE, st);
        if (g.prune_site == 0 || (qs & SOL_QS_DOWN_IN))      // (pruning elsewhere and no quantiser here: nothing to do)
            launch_prune_fq(w.a, dt, w.ra, w.perm, qs & SOL_QS_DOWN_IN, M, dff, st, g.prune_site == 0);
    }
    bool fused_down = false;
    int ns_down = 1;
    const bool q_out = (qs & SOL_QS_MLP_OUT) != 0;   // the MLP output is quantised as a whole row before the residual add
    {   // down projection (+ residual when fused)
        STAGE(ctx, ST_DOWN, st);
        if (skinny) {
            ns_down = skinny_splits((int)M, d, dff);
            if (!launch_gemm_skinny(w.a, dff, lw->w_down, d, nullptr, 0, nullptr, 0, (int)M, dff, w.big32, ns_down, st))
                return fail(ctx, SOL_ERR_UNSUPPORTED, "skinny GEMM (down): unsupported shape");
        } else {
            fused_down = mfma && !q_out && launch_gemm_resid_out(w.a, lw->w_down, w.x2, x_out, M, d, dff, st);
            if (!fused_down && !(mfma && launch_gemm_f32(w.a, lw->w_down, w.big32, d, M, d, dff, st)))
                launch_gemm_generic(w.a, dt, dff, lw->w_down, dt, dff, w.big32, d, M, d, dff, st);
        }
    }
    if (!fused_down) {   // residual
        STAGE(ctx, ST_RESID, st);
        if (q_out) launch_resid_out_fq(w.x2, w.big32, x_out, dt, w.ra, M, d, st, ns_down);
        else launch_resid_out(w.x2, w.big32, x_out, dt, M, d, st, ns_down);
    }
    return SOL_OK;
}

// Launch sequence of one decoder layer (actions already decoded into w.ra / w.perm).
static int layer_impl(sol_ctx *ctx, const sol_layer_weights *lw, const void *x_in, void *x_out, const int32_t *pos0,
                      void *kc, void *vc, int n_seq, int T, int L_max, LayerWs &w, hipStream_t st,
                      void *page_meta = nullptr, bool dense_pass = false, const PrefixView *pv = nullptr)
{
    const sol_model_cfg &g = ctx->cfg;
    const int dt = g.dtype;
    const int64_t M = (int64_t)n_seq * T;
    const int d = g.d_model, Hq = g.n_q_heads, Hkv = g.n_kv_heads, dh = g.head_dim;
    const int nq = Hq * dh, nkv = Hkv * dh, nqkv = nq + 2 * nkv;
    const uint32_t qs = g.quant_sites;

    {   // input norm + quantise (linear-input site of q/k/v)
        STAGE(ctx, ST_NORM_IN, st);
        launch_rmsnorm_fq(x_in, dt, nullptr, nullptr, lw->w_in_norm, dt, w.h, dt, w.ra, qs & SOL_QS_QKV_IN, M, d, g.rms_eps, st);
    }
    const bool mfma = dt == SOL_BF16;
    const bool skinny = use_skinny(g, M);                      // decode: HBM-bound GEMMs
    // shared prefix: the own caches hold positions P.. only; their writers get the base minus P rows
    const int crows = pv ? pv->crows : 0;
    void *kcw = pv ? (void *)((char *)kc - esize(dt) * (size_t)pv->P * dh) : kc;
    void *vcw = pv ? (void *)((char *)vc - esize(dt) * (size_t)pv->P * dh) : vc;
    bool fused_qkv = false;
    int ns_qkv = 1;
    {   // q/k/v projections (+ rotary and cache write when fused)
        STAGE(ctx, ST_QKV, st);
        if (skinny) {
            ns_qkv = skinny_splits((int)M, nqkv, d);
            if (!launch_gemm_skinny(w.h, d, lw->wq, nq, lw->wk, nkv, lw->wv, nkv, (int)M, d, w.big32, ns_qkv, st))
                return fail(ctx, SOL_ERR_UNSUPPORTED, "skinny GEMM: unsupported shape");
        } else {
            fused_qkv = mfma && launch_gemm_qkv_rope(w.h, lw->wq, lw->wk, lw->wv, w.qb, kcw, vcw, ctx->d_rope, pos0, n_seq,
                                                     T, L_max, Hq, Hkv, dh, d, ctx->d_flags, w.big32, st, crows);
            if (!fused_qkv) {
                launch_gemm_generic(w.h, dt, d, lw->wq, dt, d, w.big32, nqkv, M, nq, d, st);
                launch_gemm_generic(w.h, dt, d, lw->wk, dt, d, w.big32 + nq, nqkv, M, nkv, d, st);
                launch_gemm_generic(w.h, dt, d, lw->wv, dt, d, w.big32 + nq + nkv, nqkv, M, nkv, d, st);
            }
        }
    }
    if (!fused_qkv) {   // rotary, cache write
        STAGE(ctx, ST_ROPE, st);
        launch_rope_store(w.big32, w.qb, kcw, vcw, dt, ctx->d_rope, pos0, n_seq, T, L_max, Hq, Hkv, dh, ctx->d_flags, st,
                          ns_qkv, crows);
    }
    if (int rc = attn_stage(ctx, w, pos0, kc, vc, n_seq, T, L_max, st, page_meta, dense_pass, pv)) return rc;
    {   // quantise (o-proj input)
        STAGE(ctx, ST_QUANT_O, st);
        launch_fq_rows(w.o32, w.qb, dt, w.ra, qs & SOL_QS_O_IN, M, nq, st);
    }
    bool fused_o = false;
    int ns_o = 1;
    {   // output projection (+ residual when fused: x2 = x + attn)
        STAGE(ctx, ST_OPROJ, st);
        if (skinny) {
            ns_o = skinny_splits((int)M, d, nq);
            if (!launch_gemm_skinny(w.qb, nq, lw->wo, d, nullptr, 0, nullptr, 0, (int)M, nq, w.big32, ns_o, st))
                return fail(ctx, SOL_ERR_UNSUPPORTED, "skinny GEMM (output projection): unsupported shape");
        } else {
            fused_o = mfma && launch_gemm_resid_f32(w.qb, lw->wo, x_in, w.x2, M, d, nq, st);
            if (!fused_o) launch_gemm_generic(w.qb, dt, nq, lw->wo, dt, nq, w.big32, d, M, d, nq, st);
        }
    }
    {   // post norm (+ pruning at the MLP-input site) + quantise (gate/up input)
        STAGE(ctx, ST_NORM_POST, st);
        bool prune_in = g.prune_site == 1;
        if (prune_in) {                              // one kernel when the wave-per-row norm covers the shape
            const bool one = fused_o
                ? launch_rmsnorm_fq(w.x2, SOL_F32, nullptr, nullptr, lw->w_post_norm, dt, w.h, dt, w.ra, qs & SOL_QS_GATEUP_IN, M, d, g.rms_eps, st, 1, true)
                : launch_rmsnorm_fq(x_in, dt, w.big32, w.x2, lw->w_post_norm, dt, w.h, dt, w.ra, qs & SOL_QS_GATEUP_IN, M, d, g.rms_eps, st, ns_o, true);
            if (one) prune_in = false;               // done
        }
        // otherwise: norm to fp32, prune + quantise in place, store
        void *hdst = prune_in ? (void *)w.hn32 : w.h;
        const int hdt = prune_in ? SOL_F32 : dt;
        const bool q_here = !prune_in && (qs & SOL_QS_GATEUP_IN);
        if (g.prune_site == 1 && !prune_in) {
        } else if (fused_o)
            launch_rmsnorm_fq(w.x2, SOL_F32, nullptr, nullptr, lw->w_post_norm, dt, hdst, hdt, w.ra, q_here, M, d, g.rms_eps, st);
        else
            launch_rmsnorm_fq(x_in, dt, w.big32, w.x2, lw->w_post_norm, dt, hdst, hdt, w.ra, q_here, M, d, g.rms_eps, st, ns_o);
        if (prune_in) {
            launch_prune_fq(w.hn32, SOL_F32, w.ra, nullptr, qs & SOL_QS_GATEUP_IN, M, d, st);
            launch_fq_rows(w.hn32, w.h, dt, w.ra, false, M, d, st);
        }
    }
    if (int rc = mlp_stage(ctx, lw, w, x_out, M, skinny, st)) return rc;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ctx, SOL_ERR_HIP, std::string("kernel launch: ") + hipGetErrorString(e));
    return SOL_OK;
}

static int check_layer_weights(sol_ctx *ctx, const sol_layer_weights *w)
{
    if (!w || !w->w_in_norm || !w->wq || !w->wk || !w->wv || !w->wo || !w->w_post_norm || !w->w_gate || !w->w_up ||
        !w->w_down)
        return fail(ctx, SOL_ERR_INVALID_ARG, "a layer weight pointer is NULL");
    return SOL_OK;
}

extern "C" int sol_layer_forward(sol_ctx *ctx, const sol_layer_weights *w, const void *x_in, void *x_out,
                                 const int32_t *action_ids, const int32_t *pos0, void *k_cache, void *v_cache,
                                 int n_seq, int T, int L_max, void *workspace, size_t ws_bytes, void *stream)
{
    if (!ctx) return SOL_ERR_INVALID_ARG;
    if (n_seq < 0 || T < 0 || L_max <= 0) return fail(ctx, SOL_ERR_INVALID_ARG, "negative size");
    if (n_seq == 0 || T == 0) return SOL_OK;                        // empty batch: nothing to do
    if (int rc = check_layer_weights(ctx, w)) return rc;
    if (!x_in || !x_out || !action_ids || !k_cache || !v_cache) return fail(ctx, SOL_ERR_INVALID_ARG, "a data pointer is NULL");
    if (x_in == x_out) return fail(ctx, SOL_ERR_INVALID_ARG, "x_in and x_out must not alias");
    if (L_max > ctx->cfg.max_positions) return fail(ctx, SOL_ERR_INVALID_ARG, "L_max exceeds cfg.max_positions");
    if (T > L_max) return fail(ctx, SOL_ERR_CACHE_OVERFLOW, "T tokens cannot fit a cache of L_max positions");
    const size_t need = sol_workspace_bytes(&ctx->cfg, SOL_OP_LAYER_FORWARD, n_seq, T, L_max);
    if (!workspace || ws_bytes < need)
        return fail(ctx, SOL_ERR_WORKSPACE, "workspace too small: need " + std::to_string(need) + " bytes");
    hipStream_t st = (hipStream_t)stream;
    Carver c(workspace);
    LayerWs lw; carve_layer(c, ctx->cfg, n_seq, T, L_max, lw);
    prepare_actions(ctx, action_ids, (int64_t)n_seq * T, lw, st);
    if (T == 1 && pos0) launch_seq_order(pos0, n_seq, lw.seq_order, st);
    return layer_impl(ctx, w, x_in, x_out, pos0, k_cache, v_cache, n_seq, T, L_max, lw, st);
}

// ------------------------------------------------------------------------------------------------
// final norm + LM head + NLL
// ------------------------------------------------------------------------------------------------
static int nll_impl(sol_ctx *ctx, const sol_model_weights *mw, const void *x, int64_t M, StackWs &w,
                    const int32_t *targets, int G, int T, bool broadcast_g, float *nll_out, hipStream_t st)
{
    const sol_model_cfg &g = ctx->cfg;
    const int dt = g.dtype;
    {
        STAGE(ctx, ST_NORM_FINAL, st);
        launch_rmsnorm_fq(x, dt, nullptr, nullptr, mw->w_final_norm, dt, w.hf, dt, nullptr, false, M, g.d_model, g.rms_eps, st);
    }
    bool fused = false;
    if (dt == SOL_BF16) {   // logits stay on chip: per-tile (max, sum of exponentials), folded per row afterwards
        STAGE(ctx, ST_LMHEAD, st);
        fused = launch_gemm_nll(w.hf, mw->lm_head, targets, G, T, broadcast_g, nll_out, w.logits, M, g.vocab, g.d_model, ctx->d_flags, st);
    }
    const int64_t chunk = lm_chunk_rows(g, M);
    const size_t es = esize(dt);
    for (int64_t r0 = 0; !fused && r0 < M; r0 += chunk) {
        const int64_t rows = (M - r0 < chunk) ? M - r0 : chunk;
        {
            STAGE(ctx, ST_LMHEAD, st);
            launch_gemm_generic((const char *)w.hf + es * r0 * g.d_model, dt, g.d_model, mw->lm_head, dt, g.d_model,
                                w.logits, g.vocab, rows, g.vocab, g.d_model, st);
        }
        {
            STAGE(ctx, ST_NLL, st);
            launch_nll_rows(w.logits, rows, g.vocab, targets, r0, G, T, broadcast_g, nll_out, ctx->d_flags, st);
        }
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ctx, SOL_ERR_HIP, std::string("kernel launch: ") + hipGetErrorString(e));
    return SOL_OK;
}

// ------------------------------------------------------------------------------------------------
// decode step
// ------------------------------------------------------------------------------------------------
static int decode_step_impl(sol_ctx *ctx, const sol_model_weights *mw, const int32_t *token_ids, const void *x_in,
                            const int32_t *action_ids, const int32_t *cache_len, void *const *k_cache,
                            void *const *v_cache, void *const *page_meta, int B, int L_max, void *x_out,
                            const int32_t *targets, float *nll_out, void *workspace, size_t ws_bytes, void *stream)
{
    if (!ctx) return SOL_ERR_INVALID_ARG;
    const sol_model_cfg &g = ctx->cfg;
    if (!mw || !mw->layers) return fail(ctx, SOL_ERR_INVALID_ARG, "weights are NULL");
    for (int l = 0; l < g.n_layers; ++l)
        if (int rc = check_layer_weights(ctx, &mw->layers[l])) return rc;
    if (!token_ids && !x_in) return fail(ctx, SOL_ERR_INVALID_ARG, "token_ids and x_in are both NULL");
    if (token_ids && !mw->embed) return fail(ctx, SOL_ERR_INVALID_ARG, "token_ids given but weights->embed is NULL");
    if (!action_ids || !cache_len || !k_cache || !v_cache) return fail(ctx, SOL_ERR_INVALID_ARG, "a data pointer is NULL");
    for (int l = 0; l < g.n_layers; ++l)
        if (!k_cache[l] || !v_cache[l]) return fail(ctx, SOL_ERR_INVALID_ARG, "a per-layer cache pointer is NULL");
    if (page_meta) {
        if (g.page_size < 2 || g.dtype != SOL_BF16 || (g.head_dim != 64 && g.head_dim != 128) ||
            g.n_q_heads != 4 * g.n_kv_heads)
            return fail(ctx, SOL_ERR_UNSUPPORTED, "page metadata: needs page_size >= 2, bf16, head_dim 64/128, 4 query heads per KV head");
        for (int l = 0; l < g.n_layers; ++l)
            if (!page_meta[l]) return fail(ctx, SOL_ERR_INVALID_ARG, "a per-layer page metadata pointer is NULL");
    }
    if (nll_out && (!targets || !mw->w_final_norm || !mw->lm_head || g.vocab <= 0))
        return fail(ctx, SOL_ERR_INVALID_ARG, "nll_out needs targets, w_final_norm, lm_head and vocab > 0");
    if (B < 0 || L_max <= 0) return fail(ctx, SOL_ERR_INVALID_ARG, "negative size");
    if (L_max > g.max_positions) return fail(ctx, SOL_ERR_INVALID_ARG, "L_max exceeds cfg.max_positions");
    if (B == 0) return SOL_OK;
    const size_t need = sol_workspace_bytes(&g, SOL_OP_DECODE_STEP, B, 1, L_max);
    if (!workspace || ws_bytes < need)
        return fail(ctx, SOL_ERR_WORKSPACE, "workspace too small: need " + std::to_string(need) + " bytes");
    hipStream_t st = (hipStream_t)stream;
    Carver c(workspace);
    StackWs w; carve_stack(c, g, B, 1, false, w);
    prepare_actions(ctx, action_ids, B, w.layer, st);
    launch_seq_order(cache_len, B, w.layer.seq_order, st);
    const void *cur = x_in;
    if (token_ids) {
        launch_embed(mw->embed, token_ids, w.hf, g.dtype, B, 1, 1, g.d_model, g.vocab, ctx->d_flags, st);
        cur = w.hf;
    }
    for (int l = 0; l < g.n_layers; ++l) {
        void *dst = (l & 1) ? w.xb : w.xa;
        if (l == g.n_layers - 1 && x_out) dst = x_out;
        if (dst == cur) return fail(ctx, SOL_ERR_INVALID_ARG, "x_in and x_out must not alias");
        if (int rc = layer_impl(ctx, &mw->layers[l], cur, dst, cache_len, k_cache[l], v_cache[l], B, 1, L_max, w.layer, st,
                                page_meta ? page_meta[l] : nullptr))
            return rc;
        cur = dst;
    }
    if (nll_out) return nll_impl(ctx, mw, cur, B, w, targets, 1, 1, false, nll_out, st);
    return SOL_OK;
}

extern "C" int sol_decode_step(sol_ctx *ctx, const sol_model_weights *mw, const int32_t *token_ids, const void *x_in,
                               const int32_t *action_ids, const int32_t *cache_len, void *const *k_cache,
                               void *const *v_cache, int B, int L_max, void *x_out, const int32_t *targets,
                               float *nll_out, void *workspace, size_t ws_bytes, void *stream)
{
    return decode_step_impl(ctx, mw, token_ids, x_in, action_ids, cache_len, k_cache, v_cache, nullptr, B, L_max, x_out,
                            targets, nll_out, workspace, ws_bytes, stream);
}

extern "C" size_t sol_static_scratch_bytes(void) { return SOL_STATIC_SCRATCH_BYTES; }

extern "C" int sol_decode_step_static(sol_ctx *ctx, const sol_model_weights *mw, const int32_t *token_ids, const void *x_in,
                                      const int32_t *action_ids, const int32_t *cache_len, void *const *k_cache,
                                      void *const *v_cache, int B, int L_max, void *x_out, const int32_t *targets,
                                      float *nll_out, void *stream)
{
    if (!ctx) return SOL_ERR_INVALID_ARG;
    if (B < 0 || L_max <= 0) return fail(ctx, SOL_ERR_INVALID_ARG, "negative size");
    int dev = -1;
    SOL_HIP(ctx, hipGetDevice(&dev));
    if (dev != ctx->device)
        return fail(ctx, SOL_ERR_INVALID_ARG, "the context was created on device " + std::to_string(ctx->device) +
                                              ", the current device is " + std::to_string(dev));
    const size_t need = B > 0 ? sol_workspace_bytes(&ctx->cfg, SOL_OP_DECODE_STEP, B, 1, L_max) : 0;
    if (need > SOL_STATIC_SCRATCH_BYTES)
        return fail(ctx, SOL_ERR_WORKSPACE, "the step needs " + std::to_string(need) + " bytes of scratch, the static array holds " +
                                            std::to_string(SOL_STATIC_SCRATCH_BYTES) + ": use sol_decode_step with a workspace");
    return decode_step_impl(ctx, mw, token_ids, x_in, action_ids, cache_len, k_cache, v_cache, nullptr, B, L_max, x_out,
                            targets, nll_out, ctx->static_scratch, SOL_STATIC_SCRATCH_BYTES, stream);
}

extern "C" int sol_decode_step_paged(sol_ctx *ctx, const sol_model_weights *mw, const int32_t *token_ids, const void *x_in,
                                     const int32_t *action_ids, const int32_t *cache_len, void *const *k_cache,
                                     void *const *v_cache, void *const *page_meta, int B, int L_max, void *x_out,
                                     const int32_t *targets, float *nll_out, void *workspace, size_t ws_bytes,
                                     void *stream)
{
    if (!ctx) return SOL_ERR_INVALID_ARG;
    if (!page_meta) return fail(ctx, SOL_ERR_INVALID_ARG, "page_meta is NULL");
    return decode_step_impl(ctx, mw, token_ids, x_in, action_ids, cache_len, k_cache, v_cache, page_meta, B, L_max, x_out,
                            targets, nll_out, workspace, ws_bytes, stream);
}

extern "C" size_t sol_page_meta_bytes(const sol_model_cfg *cfg, int n_seq, int L_max)
{
    if (!cfg || cfg->page_size < 2 || n_seq <= 0 || L_max <= 0) return 0;
    const size_t pages = (size_t)(L_max + cfg->page_size - 1) / cfg->page_size;
    return (size_t)n_seq * cfg->n_kv_heads * pages * 2 * cfg->head_dim * esize(cfg->dtype);
}

extern "C" int sol_page_meta_build(sol_ctx *ctx, const void *k_cache, const int32_t *cache_len, int n_seq, int L_max,
                                   void *page_meta, void *stream)
{
    if (!ctx) return SOL_ERR_INVALID_ARG;
    const sol_model_cfg &g = ctx->cfg;
    if (!k_cache || !cache_len || !page_meta) return fail(ctx, SOL_ERR_INVALID_ARG, "a data pointer is NULL");
    if (n_seq < 0 || L_max <= 0) return fail(ctx, SOL_ERR_INVALID_ARG, "negative size");
    if (g.dtype != SOL_BF16 ||
        !launch_page_meta_build(k_cache, cache_len, page_meta, n_seq, L_max, g.n_kv_heads, g.head_dim, g.page_size,
                                (hipStream_t)stream))
        return fail(ctx, SOL_ERR_UNSUPPORTED, "page metadata: needs page_size >= 2, bf16, head_dim 64/128");
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ctx, SOL_ERR_HIP, std::string("kernel launch: ") + hipGetErrorString(e));
    return SOL_OK;
}

extern "C" int sol_kv_refresh(sol_ctx *ctx, const sol_model_weights *mw, const int32_t *token_ids, const void *x_in,
                              const int32_t *pos0, void *const *k_cache, void *const *v_cache, void *const *page_meta,
                              int n_seq, int T, int L_max, void *x_out, void *workspace, size_t ws_bytes, void *stream)
{
    if (!ctx) return SOL_ERR_INVALID_ARG;
    const sol_model_cfg &g = ctx->cfg;
    if (!mw || !mw->layers) return fail(ctx, SOL_ERR_INVALID_ARG, "weights are NULL");
    for (int l = 0; l < g.n_layers; ++l)
        if (int rc = check_layer_weights(ctx, &mw->layers[l])) return rc;
    if (n_seq < 0 || T < 0 || L_max <= 0) return fail(ctx, SOL_ERR_INVALID_ARG, "negative size");
    if ((int64_t)n_seq * T == 0) return SOL_OK;                // nothing to refresh (pointers may be NULL then)
    if (!token_ids && !x_in) return fail(ctx, SOL_ERR_INVALID_ARG, "token_ids and x_in are both NULL");
    if (token_ids && !mw->embed) return fail(ctx, SOL_ERR_INVALID_ARG, "token_ids given but weights->embed is NULL");
    if (!pos0 || !k_cache || !v_cache) return fail(ctx, SOL_ERR_INVALID_ARG, "a data pointer is NULL");
    for (int l = 0; l < g.n_layers; ++l)
        if (!k_cache[l] || !v_cache[l] || (page_meta && !page_meta[l]))
            return fail(ctx, SOL_ERR_INVALID_ARG, "a per-layer cache or metadata pointer is NULL");
    if (n_seq < 0 || T < 0 || L_max <= 0) return fail(ctx, SOL_ERR_INVALID_ARG, "negative size");
    if (L_max > g.max_positions) return fail(ctx, SOL_ERR_INVALID_ARG, "L_max exceeds cfg.max_positions");
    if (T > L_max) return fail(ctx, SOL_ERR_CACHE_OVERFLOW, "T tokens cannot fit a cache of L_max positions");
    if (page_meta && (g.page_size < 2 || g.dtype != SOL_BF16 || (g.head_dim != 64 && g.head_dim != 128)))
        return fail(ctx, SOL_ERR_UNSUPPORTED, "page metadata: needs page_size >= 2, bf16, head_dim 64/128");
    if ((int64_t)n_seq * T == 0) return SOL_OK;
    const size_t need = sol_workspace_bytes(&g, SOL_OP_KV_REFRESH, n_seq, T, L_max);
    if (!workspace || ws_bytes < need)
        return fail(ctx, SOL_ERR_WORKSPACE, "workspace too small: need " + std::to_string(need) + " bytes");
    hipStream_t st = (hipStream_t)stream;
    Carver c(workspace);
    LayerWs lw; carve_layer(c, g, n_seq, T, L_max, lw);
    const size_t es = esize(g.dtype);
    void *xa = c.take(es * (size_t)n_seq * T * g.d_model), *xb = c.take(es * (size_t)n_seq * T * g.d_model);
    const int64_t M = (int64_t)n_seq * T;
    {
        STAGE(ctx, ST_PREPARE, st);
        launch_dense_rows(g.prune_site ? g.d_model : g.d_ff, M, lw.ra, lw.row_bucket, st);
        if (prune_fq_wants_order(g.dtype, g.d_ff)) launch_bucket_sort(lw.row_bucket, M, ctx->n_buckets, lw.perm, lw.bucket_off, st);
        if (T == 1) launch_seq_order(pos0, n_seq, lw.seq_order, st);
    }
    const void *cur = x_in;
    if (token_ids) {
        launch_embed(mw->embed, token_ids, xa, g.dtype, n_seq, 1, T, g.d_model, g.vocab, ctx->d_flags, st);
        cur = xa;
    }
    for (int l = 0; l < g.n_layers; ++l) {
        void *dst = (cur == xa) ? xb : xa;
        if (l == g.n_layers - 1 && x_out) dst = x_out;
        if (dst == cur) return fail(ctx, SOL_ERR_INVALID_ARG, "x_in and x_out must not alias");
        if (int rc = layer_impl(ctx, &mw->layers[l], cur, dst, pos0, k_cache[l], v_cache[l], n_seq, T, L_max, lw, st, nullptr, true))
            return rc;
        if (page_meta &&
            !launch_page_meta_build(k_cache[l], pos0, page_meta[l], n_seq, L_max, g.n_kv_heads, g.head_dim, g.page_size, st, pos0, T))
            return fail(ctx, SOL_ERR_UNSUPPORTED, "page metadata: unsupported shape");
        cur = dst;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ctx, SOL_ERR_HIP, std::string("kernel launch: ") + hipGetErrorString(e));
    return SOL_OK;
}

extern "C" int sol_reward_advantages(sol_ctx *ctx, const float *nll, const int32_t *action_ids, const int32_t *eff,
                                     const float *targets, const sol_reward_cfg *rc, int B, int G, int T,
                                     float *avg_out, float *penalty_out, float *returns_out, float *signal_out,
                                     float *adv_out, void *workspace, size_t ws_bytes, void *stream)
{
    if (!ctx) return SOL_ERR_INVALID_ARG;
    if (B < 0 || G < 0 || T < 0) return fail(ctx, SOL_ERR_INVALID_ARG, "negative size");
    if ((int64_t)B * G * T == 0) return SOL_OK;                // nothing to reduce (pointers may be NULL then)
    if (!nll || !action_ids || !targets || !rc || !signal_out || !adv_out)
        return fail(ctx, SOL_ERR_INVALID_ARG, "a data pointer is NULL");
    if (!(rc->alpha_kappa >= 0.f) || !(rc->alpha_rho >= 0.f) || !(rc->alpha_eta >= 0.f) || !(rc->tau >= 0.f) ||
        !(rc->gamma > 0.f && rc->gamma <= 1.f) || !(rc->eps >= 0.f))
        return fail(ctx, SOL_ERR_INVALID_ARG, "reward cfg: weights, tau, eps must be >= 0 and gamma in (0, 1]");
    if (signal_out == nll || adv_out == nll || signal_out == adv_out)
        return fail(ctx, SOL_ERR_INVALID_ARG, "signal_out / adv_out must not alias nll or each other");
    if ((int64_t)B * G * T == 0) return SOL_OK;
    const size_t need = sol_workspace_bytes(&ctx->cfg, SOL_OP_REWARD, B, T, 0);
    if (!workspace || ws_bytes < need)
        return fail(ctx, SOL_ERR_WORKSPACE, "workspace too small: need " + std::to_string(need) + " bytes");
    RewardCfg r{rc->alpha_kappa, rc->alpha_rho, rc->alpha_eta, rc->tau, rc->gamma, rc->eps};
    Carver c(workspace);
    void *scratch = c.take(reward_scratch_bytes(B, T));
    launch_reward(nll, action_ids, ctx->d_table, ctx->n_actions, eff, targets, r, B, G, T, avg_out, penalty_out, returns_out,
                  signal_out, adv_out, scratch, ctx->d_flags, (hipStream_t)stream);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ctx, SOL_ERR_HIP, std::string("kernel launch: ") + hipGetErrorString(e));
    return SOL_OK;
}

// ------------------------------------------------------------------------------------------------
// teacher-forced pass over G schedules
// ------------------------------------------------------------------------------------------------
extern "C" int sol_schedule_loglik(sol_ctx *ctx, const sol_model_weights *mw, const int32_t *tokens,
                                   const int32_t *targets, const int32_t *action_ids, int B, int G, int T,
                                   float *nll_out, void *workspace, size_t ws_bytes, void *stream)
{
    if (!ctx) return SOL_ERR_INVALID_ARG;
    const sol_model_cfg &g = ctx->cfg;
    if (!mw || !mw->layers || !mw->embed || !mw->w_final_norm || !mw->lm_head)
        return fail(ctx, SOL_ERR_INVALID_ARG, "weights are NULL");
    for (int l = 0; l < g.n_layers; ++l)
        if (int rc = check_layer_weights(ctx, &mw->layers[l])) return rc;
    if (!tokens || !targets || !action_ids || !nll_out) return fail(ctx, SOL_ERR_INVALID_ARG, "a data pointer is NULL");
    if (B < 0 || G < 0 || T < 0) return fail(ctx, SOL_ERR_INVALID_ARG, "negative size");
    if (g.vocab <= 0) return fail(ctx, SOL_ERR_INVALID_ARG, "vocab must be positive");
    if (T > g.max_positions) return fail(ctx, SOL_ERR_INVALID_ARG, "T exceeds cfg.max_positions");
    if ((int64_t)B * G * T == 0) return SOL_OK;
    const int N = B * G;
    const size_t need = sol_workspace_bytes(&g, SOL_OP_SCHEDULE_LOGLIK, N, T, T);
    if (!workspace || ws_bytes < need)
        return fail(ctx, SOL_ERR_WORKSPACE, "workspace too small: need " + std::to_string(need) + " bytes");
    hipStream_t st = (hipStream_t)stream;
    Carver c(workspace);
    StackWs w; carve_stack(c, g, N, T, true, w);
    const int64_t M = (int64_t)N * T;
    prepare_actions(ctx, action_ids, M, w.layer, st);          // one plan, reused by every layer
    {
        STAGE(ctx, ST_EMBED, st);
        launch_embed(mw->embed, tokens, w.xa, g.dtype, B, G, T, g.d_model, g.vocab, ctx->d_flags, st);
    }
    void *cur = w.xa, *nxt = w.xb;
    for (int l = 0; l < g.n_layers; ++l) {
        if (int rc = layer_impl(ctx, &mw->layers[l], cur, nxt, nullptr, w.kc, w.vc, N, T, T, w.layer, st)) return rc;
        std::swap(cur, nxt);
    }
    return nll_impl(ctx, mw, cur, M, w, targets, G, T, true, nll_out, st);
}

// ------------------------------------------------------------------------------------------------
// episode pass: dense prefill once per input, then K schedules of T controlled steps on top of it
// ------------------------------------------------------------------------------------------------
struct EpisodeWs {
    bool twoseg;                           // the schedules read the prefix caches in place (no per-schedule copies)
    LayerWs pre, suf;
    void *pxa, *pxb, *pkc, *pvc;          // prefix activations (ping-pong) and one layer's prefix cache
    StackWs st;                            // suffix activations, one layer's caches, LM head scratch
    int32_t *pos0;
};

static void carve_episode_as(Carver &c, const sol_model_cfg &g, int64_t B, int64_t K, int64_t P, int64_t T, bool twoseg,
                             EpisodeWs &w)
{
    const size_t es = esize(g.dtype);
    const int64_t N = B * K, M = N * T;
    w.twoseg = twoseg;
    carve_layer(c, g, B, P, (int)P, w.pre);
    w.pxa = c.take(es * B * P * g.d_model);
    w.pxb = c.take(es * B * P * g.d_model);
    const size_t pc = es * B * g.n_kv_heads * P * g.head_dim;
    w.pkc = c.take(pc);
    w.pvc = c.take(pc);
    carve_layer(c, g, N, T, (int)(twoseg ? T : P + T), w.suf);
    w.st.xa = c.take(es * M * g.d_model);
    w.st.xb = c.take(es * M * g.d_model);
    w.st.hf = c.take(es * gemm_nll_hf_rows(M) * g.d_model);
    const size_t sc = es * N * g.n_kv_heads * (twoseg ? T : P + T) * g.head_dim;
    w.st.kc = c.take(sc);
    w.st.vc = c.take(sc);
    size_t head_bytes = 4 * lm_chunk_rows(g, M) * (size_t)(g.vocab > 0 ? g.vocab : 1);
    if (g.dtype == SOL_BF16 && g.vocab > 0 && g.vocab % 256 == 0 && gemm_nll_scratch_bytes(M, g.vocab) > head_bytes)
        head_bytes = gemm_nll_scratch_bytes(M, g.vocab);
    w.st.logits = (float *)c.take(head_bytes);
    w.pos0 = (int32_t *)c.take(4 * N);
}

// The in-place layout is taken when the tiled kernels cover the shape with two-segment addressing (that depends on
// sizes and on the distances inside the workspace only, so sizing and running agree); otherwise every schedule
// gets a copy of the prefix cache.
static void carve_episode(Carver &c, const sol_model_cfg &g, int64_t B, int64_t K, int64_t P, int64_t T, EpisodeWs &w,
                          bool copy_forced = false)
{
    const bool plain = g.page_size == 1 && g.n_sink == 0 && g.n_window == 0;
    bool twoseg = !copy_forced && g.dtype == SOL_BF16 && (plain || g.page_size > 1) && T >= 16 && P % 64 == 0 &&
                  P + T <= 4096;
    if (twoseg) {
        Carver trial((void *)(uintptr_t)(1u << 20));       // never dereferenced: only the distances between the pieces count
        EpisodeWs t;
        carve_episode_as(trial, g, B, K, P, T, true, t);
        PrefixView pv;
        pv.k = (const bf16_t *)t.pkc; pv.P = (int)P; pv.K = (int)K; pv.crows = (int)T;
        const int64_t M = B * K * T;
        const int nqkv = (g.n_q_heads + 2 * g.n_kv_heads) * g.head_dim;
        twoseg = t.suf.vt && t.pre.vt &&
                 (plain ? attn_tile_prefix_ok(t.st.kc, (int)(B * K), (int)T, g.n_q_heads, g.n_kv_heads, g.head_dim, pv)
                        : t.suf.pm && t.pre.pm &&
                          attn_tile_pages_prefix_ok((int)(B * K), (int)T, g.n_q_heads, g.n_kv_heads, g.head_dim, g.page_size, pv) &&
                          attn_tile_pages_sel_bytes(M, g.n_q_heads, (int)(P + T), g.page_size) <= 4 * (size_t)M * nqkv);
    }
    carve_episode_as(c, g, B, K, P, T, twoseg, w);
}

static size_t episode_ws_bytes(const sol_model_cfg *cfg, int B, int K, int P, int T, bool copy_forced)
{
    if (!cfg || B <= 0 || K <= 0 || P <= 0 || T <= 0) return 0;
    Carver c(nullptr);
    EpisodeWs w; carve_episode(c, *cfg, B, K, P, T, w, copy_forced);
    return c.off + 256;
}

extern "C" size_t sol_episode_workspace_bytes(const sol_model_cfg *cfg, int B, int K, int P, int T)
{
    return episode_ws_bytes(cfg, B, K, P, T, false);
}

extern "C" size_t sol_test_episode_copies_workspace_bytes(const sol_model_cfg *cfg, int B, int K, int P, int T)
{
    return episode_ws_bytes(cfg, B, K, P, T, true);
}

static int episode_impl(sol_ctx *ctx, const sol_model_weights *mw, const int32_t *prefix_tokens,
                        const int32_t *tokens, const int32_t *targets, const int32_t *action_ids, int B, int K,
                        int P, int T, float *nll_out, void *workspace, size_t ws_bytes, void *stream, bool copy_forced)
{
    if (!ctx) return SOL_ERR_INVALID_ARG;
    const sol_model_cfg &g = ctx->cfg;
    if (!mw || !mw->layers || !mw->embed || !mw->w_final_norm || !mw->lm_head)
        return fail(ctx, SOL_ERR_INVALID_ARG, "weights are NULL");
    for (int l = 0; l < g.n_layers; ++l)
        if (int rc = check_layer_weights(ctx, &mw->layers[l])) return rc;
    if (B < 0 || K < 0 || T < 0 || P <= 0) return fail(ctx, SOL_ERR_INVALID_ARG, "negative size or empty prefix");
    if ((int64_t)B * K * T == 0) return SOL_OK;                // no controlled step (pointers may be NULL then)
    if (!prefix_tokens || !tokens || !targets || !action_ids || !nll_out)
        return fail(ctx, SOL_ERR_INVALID_ARG, "a data pointer is NULL");
    if (g.vocab <= 0) return fail(ctx, SOL_ERR_INVALID_ARG, "vocab must be positive");
    if ((int64_t)P + T > g.max_positions) return fail(ctx, SOL_ERR_INVALID_ARG, "P + T exceeds cfg.max_positions");
    if ((g.head_dim * esize(g.dtype)) % 16) return fail(ctx, SOL_ERR_UNSUPPORTED, "head rows must be a multiple of 16 bytes");
    if ((int64_t)B * K * T == 0) return SOL_OK;
    const size_t need = episode_ws_bytes(&g, B, K, P, T, copy_forced);
    if (!workspace || ws_bytes < need)
        return fail(ctx, SOL_ERR_WORKSPACE, "workspace too small: need " + std::to_string(need) + " bytes");
    hipStream_t st = (hipStream_t)stream;
    Carver c(workspace);
    EpisodeWs w; carve_episode(c, g, B, K, P, T, w, copy_forced);
    const int N = B * K, L = P + T;
    const int64_t Mp = (int64_t)B * P, M = (int64_t)N * T;
    {   // plans: the prefix runs dense, the suffix under its schedules
        STAGE(ctx, ST_PREPARE, st);
        launch_dense_rows(g.prune_site ? g.d_model : g.d_ff, Mp, w.pre.ra, w.pre.row_bucket, st);
        if (prune_fq_wants_order(g.dtype, g.d_ff)) launch_bucket_sort(w.pre.row_bucket, Mp, ctx->n_buckets, w.pre.perm, w.pre.bucket_off, st);
        launch_fill_i32(w.pos0, P, N, st);
    }
    prepare_actions(ctx, action_ids, M, w.suf, st);
    {
        STAGE(ctx, ST_EMBED, st);
        launch_embed(mw->embed, prefix_tokens, w.pxa, g.dtype, B, 1, P, g.d_model, g.vocab, ctx->d_flags, st);
        launch_embed(mw->embed, tokens, w.st.xa, g.dtype, B, K, T, g.d_model, g.vocab, ctx->d_flags, st);
    }
    void *pcur = w.pxa, *pnxt = w.pxb, *cur = w.st.xa, *nxt = w.st.xb;
    for (int l = 0; l < g.n_layers; ++l) {
        // layer l of the prefix (dense, once per input) fills the prefix cache; every schedule starts from a copy
        if (int rc = layer_impl(ctx, &mw->layers[l], pcur, pnxt, nullptr, w.pkc, w.pvc, B, P, P, w.pre, st, nullptr, true)) return rc;
        std::swap(pcur, pnxt);
        if (w.twoseg) {   // the schedules read the prefix K (and the transposed V the prefix pass left in its workspace) in place
            PrefixView pv;
            pv.k = (const bf16_t *)w.pkc; pv.vt = (const bf16_t *)w.pre.vt;
            pv.P = P; pv.K = K; pv.lpadv = attn_tile_lpadv(P); pv.crows = T;
            if (g.page_size <= 1 && P + T > 1024 && w.pre.kf && launch_attn_frag_k(w.pkc, w.pre.kf, nullptr, B, P, P, g.n_kv_heads, g.head_dim, st))
                pv.kf = (const bf16_t *)w.pre.kf;     // long rows: the threshold kernel reads the prefix keys in operand order
            if (g.page_size > 1) {   // page rule: the prefix keys' metadata rows, once per input (the dense prefix pass has no use for them)
                if (!launch_page_prefix_meta(w.pkc, w.pre.pm, B, P, g.n_kv_heads, g.head_dim, g.page_size, st))
                    return fail(ctx, SOL_ERR_UNSUPPORTED, "shared-prefix attention: page size outside the tiled kernels");
                pv.pm = (const bf16_t *)w.pre.pm;
            }
            if (int rc = layer_impl(ctx, &mw->layers[l], cur, nxt, w.pos0, w.st.kc, w.st.vc, N, T, L, w.suf, st, nullptr, false, &pv))
                return rc;
        } else {
            launch_bcast_prefix(w.pkc, w.st.kc, N, K, g.n_kv_heads, P, L, g.head_dim, esize(g.dtype), st);
            launch_bcast_prefix(w.pvc, w.st.vc, N, K, g.n_kv_heads, P, L, g.head_dim, esize(g.dtype), st);
            if (int rc = layer_impl(ctx, &mw->layers[l], cur, nxt, w.pos0, w.st.kc, w.st.vc, N, T, L, w.suf, st)) return rc;
        }
        std::swap(cur, nxt);
    }
    return nll_impl(ctx, mw, cur, M, w.st, targets, K, T, true, nll_out, st);
}

extern "C" int sol_episode_loglik(sol_ctx *ctx, const sol_model_weights *mw, const int32_t *prefix_tokens,
                                  const int32_t *tokens, const int32_t *targets, const int32_t *action_ids, int B, int K,
                                  int P, int T, float *nll_out, void *workspace, size_t ws_bytes, void *stream)
{
    return episode_impl(ctx, mw, prefix_tokens, tokens, targets, action_ids, B, K, P, T, nll_out, workspace, ws_bytes, stream,
                        false);
}

extern "C" int sol_test_episode_loglik_copies(sol_ctx *ctx, const sol_model_weights *mw, const int32_t *prefix_tokens,
                                              const int32_t *tokens, const int32_t *targets, const int32_t *action_ids,
                                              int B, int K, int P, int T, float *nll_out, void *workspace, size_t ws_bytes,
                                              void *stream)
{
    return episode_impl(ctx, mw, prefix_tokens, tokens, targets, action_ids, B, K, P, T, nll_out, workspace, ws_bytes, stream,
                        true);
}

// ------------------------------------------------------------------------------------------------
// unit hooks
// ------------------------------------------------------------------------------------------------
// Arguments every stage hook shares with sol_layer_forward.
static int check_stage_args(sol_ctx *ctx, int n_seq, int T, int L_max, const void *workspace, size_t ws_bytes)
{
    if (n_seq < 0 || T < 0 || L_max <= 0) return fail(ctx, SOL_ERR_INVALID_ARG, "negative size");
    if (L_max > ctx->cfg.max_positions) return fail(ctx, SOL_ERR_INVALID_ARG, "L_max exceeds cfg.max_positions");
    if (T > L_max) return fail(ctx, SOL_ERR_CACHE_OVERFLOW, "T tokens cannot fit a cache of L_max positions");
    const size_t need = sol_workspace_bytes(&ctx->cfg, SOL_OP_LAYER_FORWARD, n_seq, T, L_max);
    if (!workspace || ws_bytes < need)
        return fail(ctx, SOL_ERR_WORKSPACE, "workspace too small: need " + std::to_string(need) + " bytes");
    return SOL_OK;
}

extern "C" int sol_test_attention_stage(sol_ctx *ctx, const void *q, const int32_t *action_ids, const int32_t *pos0,
                                        void *k_cache, void *v_cache, int n_seq, int T, int L_max, float *o_out,
                                        void *workspace, size_t ws_bytes, void *stream)
{
    if (!ctx) return SOL_ERR_INVALID_ARG;
    if (n_seq == 0 || T == 0) return SOL_OK;
    if (!q || !action_ids || !k_cache || !v_cache || !o_out) return fail(ctx, SOL_ERR_INVALID_ARG, "a data pointer is NULL");
    if (int rc = check_stage_args(ctx, n_seq, T, L_max, workspace, ws_bytes)) return rc;
    hipStream_t st = (hipStream_t)stream;
    Carver c(workspace);
    LayerWs lw; carve_layer(c, ctx->cfg, n_seq, T, L_max, lw);
    prepare_actions(ctx, action_ids, (int64_t)n_seq * T, lw, st);
    if (T == 1 && pos0) launch_seq_order(pos0, n_seq, lw.seq_order, st);
    lw.qb = const_cast<void *>(q);             // the stage only reads the queries
    lw.o32 = o_out;
    if (int rc = attn_stage(ctx, lw, pos0, k_cache, v_cache, n_seq, T, L_max, st, nullptr, false, nullptr)) return rc;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ctx, SOL_ERR_HIP, std::string("kernel launch: ") + hipGetErrorString(e));
    return SOL_OK;
}

extern "C" int sol_test_mlp_stage(sol_ctx *ctx, const sol_layer_weights *w, const void *h2, const float *x2,
                                  const int32_t *action_ids, int n_seq, int T, void *a_out, void *x_out,
                                  void *workspace, size_t ws_bytes, void *stream)
{
    if (!ctx) return SOL_ERR_INVALID_ARG;
    if (n_seq == 0 || T == 0) return SOL_OK;
    if (!w || !w->w_gate || !w->w_up || !w->w_down) return fail(ctx, SOL_ERR_INVALID_ARG, "an MLP weight pointer is NULL");
    if (!h2 || !x2 || !action_ids || !x_out) return fail(ctx, SOL_ERR_INVALID_ARG, "a data pointer is NULL");
    if (int rc = check_stage_args(ctx, n_seq, T, T > 0 ? T : 1, workspace, ws_bytes)) return rc;
    hipStream_t st = (hipStream_t)stream;
    const int64_t M = (int64_t)n_seq * T;
    Carver c(workspace);
    LayerWs lw; carve_layer(c, ctx->cfg, n_seq, T, T, lw);
    prepare_actions(ctx, action_ids, M, lw, st);
    lw.h = const_cast<void *>(h2);             // read only from here on
    lw.x2 = const_cast<float *>(x2);
    if (a_out) lw.a = a_out;
    if (int rc = mlp_stage(ctx, w, lw, x_out, M, use_skinny(ctx->cfg, M), st)) return rc;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ctx, SOL_ERR_HIP, std::string("kernel launch: ") + hipGetErrorString(e));
    return SOL_OK;
}

static int launch_status()
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { g_create_err = std::string("kernel launch: ") + hipGetErrorString(e); return SOL_ERR_HIP; }
    return SOL_OK;
}

extern "C" int sol_test_topk_select(const float *scores, int rows, int n_cols, const int32_t *n_valid, const int32_t *k,
                                    uint8_t *keep_out, void *stream)
{
    if (rows < 0 || n_cols < 0) return SOL_ERR_INVALID_ARG;
    if (rows == 0 || n_cols == 0) return SOL_OK;
    if (!scores || !n_valid || !k || !keep_out) return SOL_ERR_INVALID_ARG;
    launch_test_topk(scores, rows, n_cols, n_valid, k, keep_out, (hipStream_t)stream);
    return launch_status();
}

extern "C" int sol_test_attn_threshold(const float *scores, int rows, int n_cols, const int32_t *n_valid, const int32_t *k,
                                       uint8_t *keep_out, void *stream)
{
    if (rows < 0 || n_cols < 0) return SOL_ERR_INVALID_ARG;
    if (rows == 0 || n_cols == 0) return SOL_OK;
    if (!scores || !n_valid || !k || !keep_out) return SOL_ERR_INVALID_ARG;
    if (!launch_test_attn_threshold(scores, rows, n_cols, n_valid, k, keep_out, (hipStream_t)stream)) return SOL_ERR_UNSUPPORTED;
    return launch_status();
}

extern "C" int sol_test_gemm(const void *a, const void *w, float *c, int M, int N, int K, void *stream)
{
    if (M < 0 || N <= 0 || K <= 0) return SOL_ERR_INVALID_ARG;
    if (M == 0) return SOL_OK;
    if (!a || !w || !c) return SOL_ERR_INVALID_ARG;
    if (!launch_gemm_f32(a, w, c, N, M, N, K, (hipStream_t)stream)) return SOL_ERR_UNSUPPORTED;
    return launch_status();
}

extern "C" int sol_test_prune_mask(const float *a, int rows, int n, const int32_t *m, uint8_t *keep_out, void *stream)
{
    if (rows < 0 || n < 0) return SOL_ERR_INVALID_ARG;
    if (rows == 0 || n == 0) return SOL_OK;
    if (!a || !m || !keep_out) return SOL_ERR_INVALID_ARG;
    launch_test_prune(a, rows, n, m, keep_out, (hipStream_t)stream);
    return launch_status();
}

extern "C" int sol_test_prune_quant(void *a, int dtype, int rows, int n, const int32_t *m, const int32_t *bits,
                                    void *scratch, size_t scratch_bytes, void *stream)
{
    if (rows < 0 || n < 0 || (dtype != SOL_F32 && dtype != SOL_BF16)) return SOL_ERR_INVALID_ARG;
    if (rows == 0 || n == 0) return SOL_OK;
    if (!a || !m || !bits || !scratch) return SOL_ERR_INVALID_ARG;
    if (scratch_bytes < (size_t)rows * sizeof(RowAct)) return SOL_ERR_WORKSPACE;
    if ((size_t)n * 4 > 60 * 1024) return SOL_ERR_UNSUPPORTED;
    launch_test_prune_quant(a, dtype, rows, n, m, bits, scratch, (hipStream_t)stream);
    return launch_status();
}

extern "C" int sol_test_quant_codes(const float *z, int rows, int n, const int32_t *bits, int32_t *codes_out,
                                    float *scale_out, float *zhat_out, void *stream)
{
    if (rows < 0 || n < 0) return SOL_ERR_INVALID_ARG;
    if (rows == 0 || n == 0) return SOL_OK;
    if (!z || !bits || !codes_out || !scale_out || !zhat_out) return SOL_ERR_INVALID_ARG;
    launch_test_quant(z, rows, n, bits, codes_out, scale_out, zhat_out, (hipStream_t)stream);
    return launch_status();
}
