// C ABI of libtlt (see include/tlt.h): argument validation, workspace carving, and the sequence of
// kernel launches that makes up each of the four calls of the speculative-decoding step.
#include "../../include/tlt.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <functional>
#include <map>
#include <new>
#include <vector>

#include "kernels.h"

using namespace tlt;

namespace {

enum { CLS_GEMM = 0, CLS_ATTN = 1, CLS_COMMIT = 2, CLS_OTHER = 3, CLS_GEMM_DRAFT = 4, CLS_ATTN_DRAFT = 5, CLS_N = 6 };

struct ProfRec {
    int cls;
    double flops, bytes;
};

struct Plan {  // byte offsets into the workspace
    size_t x, xn, qkv, parts, att, g, u, act, logits, argmax, feat, top_tok, top_logp, pool_token, pool_score, pool_parent,
        pool_depth, pool_mask, fr_token, fr_src, fr_pool, fr_mask, row_map, attn_ws, accept_ws, topk_ws, status, total;
    size_t attn_ws_bytes, parts_bytes;
    int max_rows, pool_cap, feat_rows;
};

size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }

constexpr int kMaxProvisionalRows = 128;   // rows of one expansion past the committed drafter entries (two mask words)

bool plan_workspace(const tlt_model_cfg& c, int B, int n, int D, int K, int max_ctx, Plan& p) {
    if (B < 1 || n < 1 || n > TLT_MAX_TREE || D < 0 || D > TLT_MAX_DEPTH || K < 1 || K > TLT_MAX_TOPK || max_ctx < 1)
        return false;
    const size_t esz = c.dtype == TLT_F32 ? 4 : 2;
    const size_t R = (size_t)B * std::max(n, K);
    const size_t h = c.hidden, F = c.mlp, V = c.vocab;
    const size_t qkv_dim = (size_t)(c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
    p.max_rows = (int)R;
    p.pool_cap = K + std::max(0, D - 1) * K * K;
    // feature rows per sequence: the root's + one per drafter row of an expansion (deterministic:
    // K per level after the first; sampled: one per template node with children, fewer than n)
    p.feat_rows = std::max(1 + std::max(0, D - 1) * K, n);
    size_t o = 0;
    auto take = [&](size_t bytes) {
        size_t at = o;
        o = align_up(o + bytes);
        return at;
    };
    p.x = take(R * h * 4);
    p.xn = take(R * 2 * h * esz);
    p.qkv = take(R * qkv_dim * esz);
    // fp32 partial products of the projections whose sum joins the fp32 residual stream (or feeds the rotary kernel)
    // (room for four slices of the widest product at the largest row count; a plan with more cuts than fit is not taken)
    p.parts_bytes = std::max(c.dtype == TLT_BF16 ? gemm_parts_max_bytes() : (size_t)0, (c.dtype == TLT_BF16 ? 4 : 1) * R * std::max(h, qkv_dim) * 4);
    p.parts = take(p.parts_bytes);
    p.att = take(R * (size_t)c.n_q_heads * c.head_dim * esz);
    p.g = take(R * F * esz);
    p.u = take(R * F * esz);
    p.act = take(R * F * esz);
    p.logits = take(R * V * 4);
    p.argmax = take(R * 4);
    p.feat = take((size_t)B * p.feat_rows * h * 4);
    p.top_tok = take((size_t)B * K * K * 4);
    p.top_logp = take((size_t)B * K * K * 4);
    p.pool_token = take((size_t)B * p.pool_cap * 4);
    p.pool_score = take((size_t)B * p.pool_cap * 4);
    p.pool_parent = take((size_t)B * p.pool_cap * 4);
    p.pool_depth = take((size_t)B * p.pool_cap * 4);
    p.pool_mask = take((size_t)B * p.pool_cap * 16);
    const size_t FRN = (size_t)B * std::max(n, K);   // rows of one drafter pass
    p.fr_token = take(FRN * 4);
    p.fr_src = take(FRN * 4);
    p.fr_pool = take(FRN * 4);
    p.fr_mask = take(FRN * 16);
    p.row_map = take((size_t)B * 4);
    p.attn_ws_bytes = attention_workspace_bytes(B, std::max(n, K), c.n_q_heads, c.n_kv_heads, c.head_dim, max_ctx);
    p.attn_ws = take(p.attn_ws_bytes);
    p.accept_ws = take(accept_sample_workspace_bytes(B, c.vocab));
    p.topk_ws = take(row_topk_workspace_bytes(B * K, c.vocab, K));
    p.status = take(256);   // device-side status word (see tlt_device_status)
    p.total = o;
    return true;
}

bool cfg_ok(const tlt_model_cfg* c) {
    if (!c) return false;
    if (c->n_layers < 1 || c->hidden < 4 || c->hidden % 4 || c->n_q_heads < 1 || c->n_kv_heads < 1 ||
        c->n_q_heads % c->n_kv_heads || c->head_dim < 64 || c->head_dim % 64 || c->head_dim > 256 || c->mlp < 1 ||
        c->vocab < 1 || c->page_size < 1 || !(c->rms_eps > 0.f) || !(c->rope_theta > 0.f))
        return false;
    if (c->dtype != TLT_F32 && c->dtype != TLT_BF16) return false;
    // 16-byte row chunks in the cache and the activations
    const int esz = c->dtype == TLT_F32 ? 4 : 2;
    if ((c->head_dim * esz) % 16) return false;
    return true;
}

}  // namespace

struct tlt_ctx {
    tlt_model_cfg cfg;
    tlt_weights target, draft;
    std::vector<tlt_layer_weights> target_layers, draft_layers;
    bool have_draft = false;
    int max_batch, max_n, max_depth, max_topk, max_ctx;
    char* ws = nullptr;
    Plan plan;
    int hip_error = 0;
    int attn_impl = -1;  // -1: pick by dtype/shape
    bool oproj_f32 = true;   // the output projection's product reaches the residual stream unrounded
    // partial products in the workspace that the residual stream x has not absorbed yet: x (+)= their sum, formed
    // by the next kernel that reads x (in the fixed order of the slices: the result is the same on every run)
    int pending_parts = 0;
    bool pending_assign = false;
    bool in_draft = false;  // launches are accounted to the drafter's classes
    bool status_ready = false;   // the status word in the (caller-owned, uninitialised) workspace has been cleared
    // profiling
    bool prof_on = false;
    std::vector<hipEvent_t> events;
    std::vector<ProfRec> recs;
};

namespace {

int fail(tlt_ctx* ctx, hipError_t e) {
    if (ctx) ctx->hip_error = (int)e;
    return TLT_EHIP;
}

struct Scope {  // brackets one launch with events when profiling is on
    tlt_ctx* ctx;
    hipStream_t s;
    bool on;
    Scope(tlt_ctx* c, hipStream_t st, int cls, double flops, double bytes) : ctx(c), s(st), on(c && c->prof_on) {
        if (!on) return;
        size_t need = (ctx->recs.size() + 1) * 2;
        while (ctx->events.size() < need) {
            hipEvent_t ev;
            if (hipEventCreate(&ev) != hipSuccess) {
                on = false;
                return;
            }
            ctx->events.push_back(ev);
        }
        ctx->recs.push_back({cls, flops, bytes});
        (void)hipEventRecord(ctx->events[need - 2], s);
    }
    ~Scope() {
        if (on) (void)hipEventRecord(ctx->events[ctx->recs.size() * 2 - 1], s);
    }
};

#define TLT_RUN(ctx, s, cls, flops, bytes, expr)          \
    do {                                                  \
        hipError_t e__;                                   \
        {                                                 \
            Scope sc__(ctx, s, cls, flops, bytes);        \
            e__ = (expr);                                 \
        }                                                 \
        if (e__ != hipSuccess) return fail(ctx, e__);     \
    } while (0)

size_t esz_of(const tlt_ctx* c) { return c->cfg.dtype == TLT_F32 ? 4 : 2; }

int run_gemm(tlt_ctx* ctx, hipStream_t s, int out_mode, int M, int N, int K, const void* A, const void* W, void* C) {
    const double e = (double)esz_of(ctx);
    const double out_b = out_mode == OUT_T ? e : (out_mode == OUT_F32 ? 4.0 : 8.0);
    TLT_RUN(ctx, s, ctx->in_draft ? CLS_GEMM_DRAFT : CLS_GEMM, 2.0 * M * N * K, ((double)M * K + (double)N * K) * e + (double)M * N * out_b,
            gemm(s, ctx->cfg.dtype, out_mode, M, N, K, A, W, C));
    return TLT_OK;
}

unsigned int* status_word(tlt_ctx* ctx) { return (unsigned int*)(ctx->ws + ctx->plan.status); }

// The status word is cleared by the first call that may raise it (the workspace arrives uninitialised).
int ensure_status(tlt_ctx* ctx, hipStream_t s) {
    if (ctx->status_ready) return TLT_OK;
    hipError_t e = zero_f32(s, 64, (float*)status_word(ctx));
    if (e != hipSuccess) return fail(ctx, e);
    ctx->status_ready = true;
    return TLT_OK;
}

// A W^T as partial products in the workspace (see gemm_parts); returns their number through n_parts.
int run_gemm_parts(tlt_ctx* ctx, hipStream_t s, int M, int N, int K, const void* A, const void* W, int* n_parts) {
    const double e = (double)esz_of(ctx);
    hipError_t err;
    {
        Scope sc(ctx, s, ctx->in_draft ? CLS_GEMM_DRAFT : CLS_GEMM, 2.0 * M * N * K, ((double)M * K + (double)N * K) * e + (double)M * N * 4.0);
        err = gemm_parts(s, ctx->cfg.dtype, M, N, K, A, W, (float*)(ctx->ws + ctx->plan.parts), ctx->plan.parts_bytes, n_parts);
    }
    if (err != hipSuccess) return fail(ctx, err);
    return TLT_OK;
}

// x absorbs the partial products still pending (standalone: where no norm kernel follows that could do it).
int fold_pending(tlt_ctx* ctx, hipStream_t s, int M) {
    if (ctx->pending_parts == 0) return TLT_OK;
    const int h = ctx->cfg.hidden;
    TLT_RUN(ctx, s, CLS_OTHER, 0, (double)M * h * 4 * (2 + ctx->pending_parts),
            add_parts(s, (int64_t)M * h, (float*)(ctx->ws + ctx->plan.x), (const float*)(ctx->ws + ctx->plan.parts), ctx->pending_parts,
                      ctx->pending_assign));
    ctx->pending_parts = 0;
    ctx->pending_assign = false;
    return TLT_OK;
}

// out = rmsnorm(x) * gamma over the M rows of the residual stream, x first absorbing what is pending.
int norm_x(tlt_ctx* ctx, hipStream_t s, int M, const void* gamma, void* out) {
    const tlt_model_cfg& c = ctx->cfg;
    float* x = (float*)(ctx->ws + ctx->plan.x);
    const double e = (double)esz_of(ctx);
    if (ctx->pending_parts > 0) {
        const int n = ctx->pending_parts;
        const bool assign = ctx->pending_assign;
        ctx->pending_parts = 0;
        ctx->pending_assign = false;
        TLT_RUN(ctx, s, CLS_OTHER, 0, (double)M * c.hidden * (8 + 4 * n + e),
                rmsnorm_add(s, c.dtype, M, c.hidden, x, ctx->ws + ctx->plan.parts, true, gamma, c.rms_eps, out, n, assign));
    } else {
        TLT_RUN(ctx, s, CLS_OTHER, 0, (double)M * c.hidden * (4 + e), rmsnorm(s, c.dtype, M, c.hidden, x, gamma, c.rms_eps, out, nullptr));
    }
    return TLT_OK;
}

KVLayer kv_layer(const tlt_ctx* ctx, const tlt_kv* kv, int layer) {
    const tlt_model_cfg& c = ctx->cfg;
    KVLayer k;
    const size_t per_layer = (size_t)kv->n_pages * c.n_kv_heads * c.page_size * c.head_dim * esz_of(ctx);
    k.k = (char*)kv->k_pool + per_layer * layer;
    k.v = (char*)kv->v_pool + per_layer * layer;
    k.n_pages = kv->n_pages;
    k.block_table = kv->block_table;
    k.seq_len = kv->seq_len;
    k.max_pages = kv->max_pages;
    k.page_size = c.page_size;
    k.n_kv = c.n_kv_heads;
    k.d = c.head_dim;
    k.seq_len_bound = kv->seq_len_bound;
    return k;
}

// One decoder block over M = rows.B * rows.n rows whose residual stream sits in the workspace's x.
// reuse_attn_plan: the attention work list in the workspace was built by an earlier layer of the same
// forward (same rows, same sequence lengths) and is still valid.
int layer_forward(tlt_ctx* ctx, hipStream_t s, const tlt_layer_weights& w, const Rows& rows, const KVLayer& kv,
                  bool reuse_attn_plan = false) {
    const tlt_model_cfg& c = ctx->cfg;
    const Plan& p = ctx->plan;
    char* ws = ctx->ws;
    const int M = rows.B * rows.n, h = c.hidden, F = c.mlp, dt = c.dtype;
    const int q_dim = c.n_q_heads * c.head_dim, qkv_dim = q_dim + 2 * c.n_kv_heads * c.head_dim;
    const double e = (double)esz_of(ctx);
    float* x = (float*)(ws + p.x);
    int rc;
    float* parts = (float*)(ws + p.parts);
    int n_parts = 1;
    if ((rc = norm_x(ctx, s, M, w.attn_norm, ws + p.xn))) return rc;
    if (dt == TLT_BF16 && qkv_dim % 128 == 0 && (size_t)M * qkv_dim * 4 * 2 <= p.parts_bytes &&
        (M <= 256 || gemm_parts_pays(dt, M, qkv_dim, h))) {
        // too few tiles for the chip unless the projection is cut along K, which leaves fp32 partial products;
        // the rotary kernel sums them and leaves q in the model dtype (always up to 256 rows, one row of tiles;
        // above where the cost model of the cuts expects it to pay: a few hundred rows).
        if ((rc = run_gemm_parts(ctx, s, M, qkv_dim, h, ws + p.xn, w.wqkv, &n_parts))) return rc;
        TLT_RUN(ctx, s, CLS_OTHER, 0, (double)M * qkv_dim * (4 * n_parts + e),
                rope_kv_write(s, dt, rows, kv, ws + p.qkv, c.n_q_heads, c.rope_theta, w.bqkv, parts, n_parts));
    } else {
        if ((rc = run_gemm(ctx, s, OUT_T, M, qkv_dim, h, ws + p.xn, w.wqkv, ws + p.qkv))) return rc;
        TLT_RUN(ctx, s, CLS_OTHER, 0, (double)M * qkv_dim * e * 2,
                rope_kv_write(s, dt, rows, kv, ws + p.qkv, c.n_q_heads, c.rope_theta, w.bqkv));
    }
    {
        // algorithmic traffic: one pass over the cached K and V of every sequence (bounded by the
        // host-known length) plus q in / out; flops: 4 * d per (query row, head, key)
        const double keys = (double)rows.B * ((double)kv.seq_len_bound + rows.n_region);
        const double bytes = keys * 2.0 * c.n_kv_heads * c.head_dim * e + 2.0 * M * q_dim * e;
        const double flops = 4.0 * c.head_dim * c.n_q_heads * (double)rows.n * keys;
        TLT_RUN(ctx, s, ctx->in_draft ? CLS_ATTN_DRAFT : CLS_ATTN, flops, bytes,
                attention(s, dt, rows, kv, ws + p.qkv, ws + p.att, c.n_q_heads, ws + p.attn_ws, p.attn_ws_bytes, ctx->attn_impl,
                          reuse_attn_plan, ctx->status_ready ? status_word(ctx) : nullptr));
    }
    // the output projection's product (fp32, possibly several partial products of a K split) joins the
    // residual stream inside the norm kernel that follows: plain stores in the GEMM's epilogue instead of
    // a read-modify-write of the stream by every tile, and a sum formed in a fixed order
    if (dt == TLT_BF16 && !ctx->oproj_f32 && M > 256) {   // (measurement switch: the product rounded to the model dtype)
        if ((rc = run_gemm(ctx, s, OUT_T, M, h, q_dim, ws + p.att, w.wo, parts))) return rc;
        TLT_RUN(ctx, s, CLS_OTHER, 0, (double)M * h * (8 + 2 * e),
                rmsnorm_add(s, dt, M, h, x, parts, false, w.mlp_norm, c.rms_eps, ws + p.xn));
    } else {
        if ((rc = run_gemm_parts(ctx, s, M, h, q_dim, ws + p.att, w.wo, &n_parts))) return rc;
        ctx->pending_parts = n_parts;
        ctx->pending_assign = false;
        if ((rc = norm_x(ctx, s, M, w.mlp_norm, ws + p.xn))) return rc;
    }
    if (gemm_glu_supported(dt, M, F, h, ws + p.xn, w.wg, w.wu)) {
        TLT_RUN(ctx, s, ctx->in_draft ? CLS_GEMM_DRAFT : CLS_GEMM, 4.0 * M * F * h,
                ((double)M * h + 2.0 * F * h + (double)M * F) * e, gemm_glu(s, M, F, h, ws + p.xn, w.wg, w.wu, ws + p.act));
    } else {
        if ((rc = run_gemm(ctx, s, OUT_T, M, F, h, ws + p.xn, w.wg, ws + p.g))) return rc;
        if ((rc = run_gemm(ctx, s, OUT_T, M, F, h, ws + p.xn, w.wu, ws + p.u))) return rc;
        TLT_RUN(ctx, s, CLS_OTHER, 0, (double)M * F * e * 3, swiglu(s, dt, (int64_t)M * F, ws + p.g, ws + p.u, ws + p.act));
    }
    // the down projection's product stays pending: the next kernel that reads the stream absorbs it
    if ((rc = run_gemm_parts(ctx, s, M, h, F, ws + p.act, w.wd, &n_parts))) return rc;
    ctx->pending_parts = n_parts;
    ctx->pending_assign = false;
    return TLT_OK;
}

int check_kv(const tlt_ctx* ctx, const tlt_kv* kv, int new_rows) {
    if (!kv || !kv->k_pool || !kv->v_pool || !kv->block_table || !kv->seq_len || kv->n_pages < 1 || kv->max_pages < 1 ||
        kv->seq_len_bound < 0)
        return TLT_EINVAL;
    if ((int64_t)kv->seq_len_bound + new_rows > (int64_t)kv->max_pages * ctx->cfg.page_size) return TLT_ENOPAGES;
    if (kv->seq_len_bound + new_rows > ctx->max_ctx) return TLT_ESHAPE;
    return TLT_OK;
}

bool tree_ok(const tlt_tree* t) { return t && t->token && t->parent && t->depth && t->anc_mask && t->n >= 1 && t->n <= TLT_MAX_TREE; }

}  // namespace

extern "C" {

const char* tlt_strerror(int code) {
    switch (code) {
        case TLT_OK: return "ok";
        case TLT_EINVAL: return "invalid argument";
        case TLT_ESHAPE: return "size exceeds the limits given to tlt_create (or workspace too small)";
        case TLT_ENOPAGES: return "block table too short for seq_len_bound + new rows";
        case TLT_EHIP: return "HIP call failed";
        case TLT_ENOTIMPL: return "not implemented";
        case TLT_ESYNC: return "workgroups of a kernel could not meet on the device (chip busy with other work)";
        default: return "unknown error";
    }
}

int tlt_last_hip_error(const tlt_ctx* ctx) { return ctx ? ctx->hip_error : 0; }

size_t tlt_workspace_bytes(const tlt_model_cfg* cfg, int max_batch, int max_n, int max_depth, int max_topk, int max_ctx) {
    Plan p;
    if (!cfg_ok(cfg) || !plan_workspace(*cfg, max_batch, max_n, max_depth, max_topk, max_ctx, p)) return 0;
    return p.total;
}

int tlt_create(tlt_ctx** out, const tlt_model_cfg* cfg, const tlt_weights* target, const tlt_weights* draft, int max_batch,
               int max_n, int max_depth, int max_topk, int max_ctx, void* workspace, size_t workspace_bytes) {
    if (!out || !cfg_ok(cfg) || !target || !target->embed || !target->lm_head || !target->final_norm || !target->layers ||
        !workspace)
        return TLT_EINVAL;
    if (((uintptr_t)workspace & 255) != 0) return TLT_EINVAL;
    Plan p;
    if (!plan_workspace(*cfg, max_batch, max_n, max_depth, max_topk, max_ctx, p)) return TLT_EINVAL;
    if (workspace_bytes < p.total) return TLT_ESHAPE;
    for (int l = 0; l < cfg->n_layers; ++l) {
        const tlt_layer_weights& w = target->layers[l];
        if (!w.attn_norm || !w.wqkv || !w.wo || !w.mlp_norm || !w.wg || !w.wu || !w.wd) return TLT_EINVAL;
    }
    if (draft) {
        if (!draft->fc || !draft->layers) return TLT_EINVAL;
        const tlt_layer_weights& w = draft->layers[0];
        if (!w.attn_norm || !w.wqkv || !w.wo || !w.mlp_norm || !w.wg || !w.wu || !w.wd) return TLT_EINVAL;
    }
    tlt_ctx* c = new (std::nothrow) tlt_ctx();
    if (!c) return TLT_EINVAL;
    c->cfg = *cfg;
    c->target = *target;
    c->target_layers.assign(target->layers, target->layers + cfg->n_layers);
    c->target.layers = c->target_layers.data();
    if (draft) {
        c->have_draft = true;
        c->draft = *draft;
        c->draft_layers.assign(draft->layers, draft->layers + 1);
        c->draft.layers = c->draft_layers.data();
    }
    c->max_batch = max_batch;
    c->max_n = max_n;
    c->max_depth = max_depth;
    c->max_topk = max_topk;
    c->max_ctx = max_ctx;
    c->ws = (char*)workspace;
    c->plan = p;
    *out = c;
    return TLT_OK;
}

int tlt_destroy(tlt_ctx* ctx) {
    if (!ctx) return TLT_EINVAL;
    for (hipEvent_t e : ctx->events) (void)hipEventDestroy(e);
    delete ctx;
    return TLT_OK;
}

int tlt_set_attention_impl(tlt_ctx* ctx, int impl) {
    if (!ctx) return TLT_EINVAL;
    ctx->attn_impl = impl;
    return TLT_OK;
}

int tlt_device_status(tlt_ctx* ctx, void* stream, uint32_t* flags) {
    if (!ctx) return TLT_EINVAL;
    if (flags) *flags = 0;
    if (!ctx->status_ready) return TLT_OK;   // nothing that could raise it has run
    hipStream_t s = (hipStream_t)stream;
    uint32_t host = 0;
    hipError_t e = hipMemcpyAsync(&host, status_word(ctx), sizeof(host), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return fail(ctx, e);
    if (flags) *flags = host;
    if (host != 0) {
        e = zero_f32(s, 64, (float*)status_word(ctx));
        if (e != hipSuccess) return fail(ctx, e);
    }
    return (host & TLT_STATUS_CONTEXT_TRUNCATED) ? TLT_ESHAPE : ((host & TLT_STATUS_NO_RENDEZVOUS) ? TLT_ESYNC : TLT_OK);
}

int tlt_set_oproj_rounding(tlt_ctx* ctx, int round_to_model_dtype) {
    if (!ctx) return TLT_EINVAL;
    ctx->oproj_f32 = round_to_model_dtype == 0;
    return TLT_OK;
}

int tlt_tree_finalize(tlt_ctx* ctx, void* stream, int B, tlt_tree* tree) {
    if (!ctx || !tree_ok(tree) || B < 1) return TLT_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    TLT_RUN(ctx, s, CLS_OTHER, 0, 0, tree_finalize(s, B, tree->n, tree->parent, tree->depth, tree->anc_mask));
    return TLT_OK;
}

int tlt_verify_forward(tlt_ctx* ctx, void* stream, int B, const tlt_tree* tree, tlt_kv* kv, float* out_logits,
                       int32_t* out_argmax, float* out_lse, float* out_hidden) {
    if (!ctx || !tree_ok(tree) || B < 1) return TLT_EINVAL;
    if (B > ctx->max_batch || tree->n > ctx->max_n) return TLT_ESHAPE;
    int rc = check_kv(ctx, kv, tree->n);
    if (rc) return rc;
    hipStream_t s = (hipStream_t)stream;
    if ((rc = ensure_status(ctx, s))) return rc;
    ctx->pending_parts = 0;   // (nothing of an earlier call is pending: every call absorbs what it leaves)
    const tlt_model_cfg& c = ctx->cfg;
    const Plan& p = ctx->plan;
    char* ws = ctx->ws;
    const int n = tree->n, M = B * n, h = c.hidden, V = c.vocab;
    const double e = (double)esz_of(ctx);
    float* x = (float*)(ws + p.x);

    TLT_RUN(ctx, s, CLS_OTHER, 0, (double)M * h * (e + 4), embed_rows(s, c.dtype, M, h, V, tree->token, ctx->target.embed, x));
    Rows rows;
    rows.B = B;
    rows.n = n;
    rows.pos_off = tree->depth;
    rows.mask = tree->anc_mask;
    rows.mask_words = 1;
    rows.n_region = n;
    for (int l = 0; l < c.n_layers; ++l) {
        rc = layer_forward(ctx, s, ctx->target.layers[l], rows, kv_layer(ctx, kv, l), l > 0);
        if (rc) return rc;
    }
    // (the last block's down projection is still pending: the final norm absorbs it into x, or, when no logits
    // are wanted, a plain add)
    if (out_logits || out_argmax || out_lse) {
        float* logits = out_logits ? out_logits : (float*)(ws + p.logits);
        if ((rc = norm_x(ctx, s, M, ctx->target.final_norm, ws + p.xn))) return rc;
        if (out_hidden) TLT_RUN(ctx, s, CLS_OTHER, 0, (double)M * h * 8, copy_f32(s, (int64_t)M * h, x, out_hidden));
        if (!out_logits && !out_lse && gemm_argmax_supported(c.dtype, M, V, h, ws + p.xn, ctx->target.lm_head)) {
            // only the most likely tokens are wanted: the logits never leave the LM head's registers
            // (block partials go where the logits would have gone: M * V/128 * 8 bytes of M * V * 4)
            TLT_RUN(ctx, s, CLS_GEMM, 2.0 * M * V * h, ((double)M * h + (double)V * h) * e,
                    gemm_argmax(s, M, V, h, ws + p.xn, ctx->target.lm_head, logits, out_argmax));
        } else {
            if ((rc = run_gemm(ctx, s, OUT_F32, M, V, h, ws + p.xn, ctx->target.lm_head, logits))) return rc;
            if (out_argmax) TLT_RUN(ctx, s, CLS_OTHER, 0, (double)M * V * 4, row_argmax(s, M, V, logits, out_argmax, ws + p.parts, p.parts_bytes));   // (nothing is pending: the slices' buffer is idle)
            if (out_lse) TLT_RUN(ctx, s, CLS_OTHER, 0, (double)M * V * 8, row_lse(s, M, V, logits, out_lse));
        }
    } else {
        if ((rc = fold_pending(ctx, s, M))) return rc;
        if (out_hidden) TLT_RUN(ctx, s, CLS_OTHER, 0, (double)M * h * 8, copy_f32(s, (int64_t)M * h, x, out_hidden));
    }
    return TLT_OK;
}

// x = fc([embedding ; hidden]) of the drafter (2h -> h), left pending as partial products: with few rows the
// product has far fewer tiles than the chip has CUs while K = 2h is long, so it is cut along K; the
// drafter block's first norm kernel forms x from the slices.
static int draft_fc(tlt_ctx* ctx, hipStream_t s, int M, const void* xin) {
    int n_parts = 1;
    int rc = run_gemm_parts(ctx, s, M, ctx->cfg.hidden, 2 * ctx->cfg.hidden, xin, ctx->draft.fc, &n_parts);
    if (rc) return rc;
    ctx->pending_parts = n_parts;
    ctx->pending_assign = true;
    return TLT_OK;
}

// Drafter catch-up shared by both expansion modes: entries for the newly committed positions, the
// last one's output as feature row 0, committed length advanced.
static int draft_extend_rows(tlt_ctx* ctx, hipStream_t s, int B, const int32_t* new_tokens, const int32_t* new_src,
                             const int32_t* n_new, int new_stride, const float* hidden, int hidden_n, tlt_kv* draft_kv,
                             KVLayer& kvl) {
    const tlt_model_cfg& c = ctx->cfg;
    const Plan& p = ctx->plan;
    char* ws = ctx->ws;
    const int h = c.hidden, V = c.vocab, dt = c.dtype;
    const double e = (double)esz_of(ctx);
    float* x = (float*)(ws + p.x);
    float* feat = (float*)(ws + p.feat);
    const int FR = p.feat_rows;
    int rc;
    const int M = B * new_stride;
    TLT_RUN(ctx, s, CLS_OTHER, 0, (double)M * h * (4 + 3 * e),
            draft_input(s, dt, B, new_stride, h, V, new_tokens, new_src, n_new, hidden_n, (int64_t)B * hidden_n, hidden,
                        ctx->target.embed, ws + p.xn));
    if ((rc = draft_fc(ctx, s, M, ws + p.xn))) return rc;
    Rows rows;
    rows.B = B;
    rows.n = new_stride;
    rows.n_valid = n_new;
    rows.pos_stride = 1;
    rows.n_region = new_stride;
    if ((rc = layer_forward(ctx, s, ctx->draft.layers[0], rows, kvl))) return rc;
    if ((rc = fold_pending(ctx, s, M))) return rc;
    TLT_RUN(ctx, s, CLS_OTHER, 0, (double)B * h * 8, gather_last_rows(s, B, new_stride, h, n_new, x, feat, FR));
    TLT_RUN(ctx, s, CLS_OTHER, 0, 0, add_i32(s, B, draft_kv->seq_len, n_new, 0));
    kvl.seq_len_bound += new_stride;
    return TLT_OK;
}

int tlt_draft_expand(tlt_ctx* ctx, void* stream, int B, int depth, int topk, int n_verify, int mode,
                     const int32_t* new_tokens, const int32_t* new_src, const int32_t* n_new, int new_stride,
                     const float* hidden, int hidden_n, const int32_t* root_tokens, tlt_kv* draft_kv, tlt_tree* out_tree) {
    if (!ctx || !ctx->have_draft || B < 1 || depth < 0 || new_stride < 0) return TLT_EINVAL;
    if (mode != 0) return TLT_ENOTIMPL;
    const bool do_extend = new_stride > 0;
    const bool do_expand = depth >= 1 && out_tree != nullptr;
    if (do_extend && (!new_tokens || !new_src || !n_new || !hidden || hidden_n < 1)) return TLT_EINVAL;
    if (do_expand && (!tree_ok(out_tree) || !out_tree->score || (!root_tokens && !do_extend) || topk < 1 || n_verify < 1))
        return TLT_EINVAL;
    if (B > ctx->max_batch || new_stride > std::max(ctx->max_n, ctx->max_topk)) return TLT_ESHAPE;
    if (do_expand && (depth > ctx->max_depth || topk > ctx->max_topk || n_verify > ctx->max_n)) return TLT_ESHAPE;
    // a provisional drafter row is one bit of a 128-bit visibility mask
    if (do_expand && (depth - 1) * topk > kMaxProvisionalRows) return TLT_ESHAPE;
    const int pool_n = do_expand ? topk + (depth - 1) * topk * topk : 0;
    if (do_expand && out_tree->n != std::min(n_verify, 1 + pool_n)) return TLT_EINVAL;
    const int prov_rows = do_expand ? (depth - 1) * topk : 0;
    int rc = check_kv(ctx, draft_kv, new_stride + prov_rows);
    if (rc) return rc;

    struct DraftFlag {
        tlt_ctx* c;
        explicit DraftFlag(tlt_ctx* x) : c(x) { c->in_draft = true; }
        ~DraftFlag() { c->in_draft = false; }
    } draft_flag(ctx);
    hipStream_t s = (hipStream_t)stream;
    if ((rc = ensure_status(ctx, s))) return rc;
    ctx->pending_parts = 0;
    const tlt_model_cfg& c = ctx->cfg;
    const Plan& p = ctx->plan;
    char* ws = ctx->ws;
    const int h = c.hidden, V = c.vocab, dt = c.dtype;
    const double e = (double)esz_of(ctx);
    float* x = (float*)(ws + p.x);
    float* feat = (float*)(ws + p.feat);
    float* logits = (float*)(ws + p.logits);
    int32_t* top_tok = (int32_t*)(ws + p.top_tok);
    float* top_logp = (float*)(ws + p.top_logp);
    int32_t* row_map = (int32_t*)(ws + p.row_map);
    const int FR = p.feat_rows;
    const tlt_layer_weights& lw = ctx->draft.layers[0];
    KVLayer kvl = kv_layer(ctx, draft_kv, 0);

    if (do_extend && (rc = draft_extend_rows(ctx, s, B, new_tokens, new_src, n_new, new_stride, hidden, hidden_n, draft_kv, kvl)))
        return rc;
    if (!do_expand) return TLT_OK;

    DraftState st;
    st.P = p.pool_cap;
    st.pool_token = (int32_t*)(ws + p.pool_token);
    st.pool_score = (float*)(ws + p.pool_score);
    st.pool_parent = (int32_t*)(ws + p.pool_parent);
    st.pool_depth = (int32_t*)(ws + p.pool_depth);
    st.pool_mask = (uint64_t*)(ws + p.pool_mask);
    st.fr_token = (int32_t*)(ws + p.fr_token);
    st.fr_src = (int32_t*)(ws + p.fr_src);
    st.fr_pool = (int32_t*)(ws + p.fr_pool);
    st.fr_mask = (uint64_t*)(ws + p.fr_mask);

    // root distribution: feature row 0 of every sequence -> final norm -> LM head -> top-k
    TLT_RUN(ctx, s, CLS_OTHER, 0, 0, iota_scaled(s, B, row_map, FR));
    TLT_RUN(ctx, s, CLS_OTHER, 0, (double)B * h * (4 + e),
            rmsnorm(s, dt, B, h, feat, ctx->target.final_norm, c.rms_eps, ws + p.xn, row_map));
    if ((rc = run_gemm(ctx, s, OUT_F32, B, V, h, ws + p.xn, ctx->target.lm_head, logits))) return rc;
    TLT_RUN(ctx, s, CLS_OTHER, 0, (double)B * V * 4, row_topk_logp(s, B, V, topk, logits, top_tok, top_logp, ws + p.topk_ws));
    TLT_RUN(ctx, s, CLS_OTHER, 0, 0, draft_level0(s, B, topk, top_tok, top_logp, st, FR));

    for (int level = 1; level < depth; ++level) {
        const int M = B * topk;
        TLT_RUN(ctx, s, CLS_OTHER, 0, (double)M * h * (4 + 3 * e),
                draft_input(s, dt, B, topk, h, V, st.fr_token, st.fr_src, nullptr, FR, (int64_t)B * FR, feat,
                            ctx->target.embed, ws + p.xn));
        if ((rc = draft_fc(ctx, s, M, ws + p.xn))) return rc;
        Rows rows;
        rows.B = B;
        rows.n = topk;
        rows.pos_base = level - 1;
        rows.pos_stride = 0;
        rows.slot_base = (level - 1) * topk;
        rows.mask = st.fr_mask;
        rows.mask_words = 2;
        rows.n_region = level * topk;
        if ((rc = layer_forward(ctx, s, lw, rows, kvl))) return rc;
        if ((rc = norm_x(ctx, s, M, ctx->target.final_norm, ws + p.xn))) return rc;   // (absorbs the pending down projection into x)
        TLT_RUN(ctx, s, CLS_OTHER, 0, (double)M * h * 8, scatter_rows(s, M, topk, h, x, feat, FR, 1 + (level - 1) * topk));
        if ((rc = run_gemm(ctx, s, OUT_F32, M, V, h, ws + p.xn, ctx->target.lm_head, logits))) return rc;
        TLT_RUN(ctx, s, CLS_OTHER, 0, (double)M * V * 4, row_topk_logp(s, M, V, topk, logits, top_tok, top_logp, ws + p.topk_ws));
        TLT_RUN(ctx, s, CLS_OTHER, 0, 0, draft_level_select(s, B, topk, level, top_tok, top_logp, st, FR));
    }
    TLT_RUN(ctx, s, CLS_OTHER, 0, 0,
            draft_prune(s, B, pool_n, out_tree->n, root_tokens, new_tokens, n_new, new_stride, st, out_tree->token, out_tree->parent, out_tree->depth,
                        out_tree->anc_mask, out_tree->score));
    return TLT_OK;
}

int tlt_draft_pool(tlt_ctx* ctx, void* stream, int B, int depth, int topk, int32_t* token, int32_t* parent, float* score) {
    if (!ctx || !ctx->have_draft || B < 1 || depth < 1 || topk < 1 || !token || !parent || !score) return TLT_EINVAL;
    if (B > ctx->max_batch || depth > ctx->max_depth || topk > ctx->max_topk) return TLT_ESHAPE;
    hipStream_t s = (hipStream_t)stream;
    const Plan& p = ctx->plan;
    const size_t n = (size_t)topk + (size_t)(depth - 1) * topk * topk, src_pitch = (size_t)p.pool_cap * 4;
    const struct {
        void* dst;
        size_t off;
    } parts[3] = {{token, p.pool_token}, {parent, p.pool_parent}, {score, p.pool_score}};
    for (const auto& part : parts) {
        hipError_t e = hipMemcpy2DAsync(part.dst, n * 4, ctx->ws + part.off, src_pitch, n * 4, (size_t)B,
                                        hipMemcpyDeviceToDevice, s);
        if (e != hipSuccess) return fail(ctx, e);
    }
    return TLT_OK;
}

int tlt_draft_sample(tlt_ctx* ctx, void* stream, int B, int depth, int topk, int n_verify, float temperature,
                     const int32_t* new_tokens, const int32_t* new_src, const int32_t* n_new, int new_stride,
                     const float* hidden, int hidden_n, const int32_t* root_tokens, tlt_kv* draft_kv, const uint32_t* u_draw,
                     tlt_tree* out_tree, float* out_draft_q) {
    if (!ctx || !ctx->have_draft || B < 1 || depth < 1 || new_stride < 0 || topk < 1 || n_verify < 1 || !(temperature > 0.f))
        return TLT_EINVAL;
    const bool do_extend = new_stride > 0;
    if (do_extend && (!new_tokens || !new_src || !n_new || !hidden || hidden_n < 1)) return TLT_EINVAL;
    if (!tree_ok(out_tree) || !out_tree->score || (!root_tokens && !do_extend) || !u_draw || !out_draft_q) return TLT_EINVAL;
    if (B > ctx->max_batch || new_stride > std::max(ctx->max_n, ctx->max_topk)) return TLT_ESHAPE;
    if (depth > ctx->max_depth || topk > ctx->max_topk || n_verify > ctx->max_n) return TLT_ESHAPE;
    // the template and, from it, the work of every level
    int32_t t_parent[TLT_MAX_TREE], t_rank[TLT_MAX_TREE], t_depth[TLT_MAX_TREE], n = 0;
    int rc = tlt_template_build(topk, depth, n_verify, t_parent, t_rank, t_depth, &n);
    if (rc) return rc;
    if (out_tree->n != n) return TLT_EINVAL;
    int first_child[TLT_MAX_TREE], n_child[TLT_MAX_TREE] = {}, inner_idx[TLT_MAX_TREE];
    for (int i = n - 1; i >= 1; --i) {
        first_child[t_parent[i]] = i;   // children are consecutive: the last write is the lowest index
        ++n_child[t_parent[i]];
    }
    int n_inner = 0;   // nodes other than the root that have children = provisional drafter rows
    for (int i = 1; i < n; ++i) inner_idx[i] = n_child[i] ? n_inner++ : -1;
    rc = check_kv(ctx, draft_kv, new_stride + n_inner);
    if (rc) return rc;

    struct DraftFlag {
        tlt_ctx* c;
        explicit DraftFlag(tlt_ctx* x) : c(x) { c->in_draft = true; }
        ~DraftFlag() { c->in_draft = false; }
    } draft_flag(ctx);
    hipStream_t s = (hipStream_t)stream;
    if ((rc = ensure_status(ctx, s))) return rc;
    ctx->pending_parts = 0;
    const tlt_model_cfg& c = ctx->cfg;
    const Plan& p = ctx->plan;
    char* ws = ctx->ws;
    const int h = c.hidden, V = c.vocab, dt = c.dtype;
    const double e = (double)esz_of(ctx);
    float* x = (float*)(ws + p.x);
    float* feat = (float*)(ws + p.feat);
    float* logits = (float*)(ws + p.logits);
    int32_t* row_map = (int32_t*)(ws + p.row_map);
    int32_t* fr_token = (int32_t*)(ws + p.fr_token);
    int32_t* fr_src = (int32_t*)(ws + p.fr_src);
    uint64_t* fr_mask = (uint64_t*)(ws + p.fr_mask);
    const int FR = p.feat_rows;
    const tlt_layer_weights& lw = ctx->draft.layers[0];
    KVLayer kvl = kv_layer(ctx, draft_kv, 0);

    if (do_extend && (rc = draft_extend_rows(ctx, s, B, new_tokens, new_src, n_new, new_stride, hidden, hidden_n, draft_kv, kvl)))
        return rc;

    TmplParents tp;
    for (int i = 0; i < TLT_MAX_TREE; ++i) tp.parent[i] = (int8_t)(i < n ? t_parent[i] : -1);
    TLT_RUN(ctx, s, CLS_OTHER, 0, 0,
            tmpl_tree_init(s, B, n, tp, root_tokens, new_tokens, n_new, new_stride, out_tree->token, out_tree->parent,
                           out_tree->score));
    TLT_RUN(ctx, s, CLS_OTHER, 0, 0, tree_finalize(s, B, n, out_tree->parent, out_tree->depth, out_tree->anc_mask));
    if (n == 1) return TLT_OK;

    // the root's distribution (feature row 0 -> final norm -> LM head) and its children
    TmplRows lv;
    lv.R = 1;
    lv.node[0] = 0;
    lv.first_child[0] = (uint8_t)first_child[0];
    lv.n_child[0] = (uint8_t)n_child[0];
    TLT_RUN(ctx, s, CLS_OTHER, 0, 0, iota_scaled(s, B, row_map, FR));
    TLT_RUN(ctx, s, CLS_OTHER, 0, (double)B * h * (4 + e),
            rmsnorm(s, dt, B, h, feat, ctx->target.final_norm, c.rms_eps, ws + p.xn, row_map));
    if ((rc = run_gemm(ctx, s, OUT_F32, B, V, h, ws + p.xn, ctx->target.lm_head, logits))) return rc;
    TLT_RUN(ctx, s, CLS_OTHER, 0, (double)B * V * 12,
            softmax_draw(s, B, n, V, temperature, lv, logits, u_draw, out_tree->token, out_draft_q,
                         ctx->pending_parts == 0 ? ws + p.parts : nullptr, p.parts_bytes));   // (the slices' buffer is idle here)

    // level d: the nodes of depth d that have children, one drafter row each (provisional cache row
    // and feature row 1 + its index among such nodes)
    uint64_t mask_of[TLT_MAX_TREE] = {};
    for (int d = 1; d < depth; ++d) {
        lv.R = 0;
        int slot_base = -1;
        for (int i = 1; i < n; ++i) {
            if (t_depth[i] != d || !n_child[i]) continue;
            const int par = t_parent[i];
            mask_of[i] = (par > 0 ? mask_of[par] : 0ull) | (1ull << inner_idx[i]);
            if (slot_base < 0) slot_base = inner_idx[i];
            const int r = lv.R++;
            lv.node[r] = (uint8_t)i;
            lv.first_child[r] = (uint8_t)first_child[i];
            lv.n_child[r] = (uint8_t)n_child[i];
            lv.src[r] = (uint8_t)(par > 0 ? 1 + inner_idx[par] : 0);
            lv.mask[r] = mask_of[i];
        }
        if (lv.R == 0) break;
        const int M = B * lv.R;
        TLT_RUN(ctx, s, CLS_OTHER, 0, 0, tmpl_level_rows(s, B, n, lv, out_tree->token, fr_token, fr_src, fr_mask));
        TLT_RUN(ctx, s, CLS_OTHER, 0, (double)M * h * (4 + 3 * e),
                draft_input(s, dt, B, lv.R, h, V, fr_token, fr_src, nullptr, FR, (int64_t)B * FR, feat, ctx->target.embed,
                            ws + p.xn));
        if ((rc = draft_fc(ctx, s, M, ws + p.xn))) return rc;
        Rows rows;
        rows.B = B;
        rows.n = lv.R;
        rows.pos_base = d - 1;
        rows.pos_stride = 0;
        rows.slot_base = slot_base;
        rows.mask = fr_mask;
        rows.mask_words = 1;
        rows.n_region = slot_base + lv.R;
        if ((rc = layer_forward(ctx, s, lw, rows, kvl))) return rc;
        if ((rc = norm_x(ctx, s, M, ctx->target.final_norm, ws + p.xn))) return rc;   // (absorbs the pending down projection into x)
        TLT_RUN(ctx, s, CLS_OTHER, 0, (double)M * h * 8, scatter_rows(s, M, lv.R, h, x, feat, FR, 1 + slot_base));
        if ((rc = run_gemm(ctx, s, OUT_F32, M, V, h, ws + p.xn, ctx->target.lm_head, logits))) return rc;
        TLT_RUN(ctx, s, CLS_OTHER, 0, (double)M * V * 12,
                softmax_draw(s, B, n, V, temperature, lv, logits, u_draw, out_tree->token, out_draft_q,
                         ctx->pending_parts == 0 ? ws + p.parts : nullptr, p.parts_bytes));   // (the slices' buffer is idle here)
    }
    return TLT_OK;
}

int tlt_accept(tlt_ctx* ctx, void* stream, int B, int mode, float temperature, const tlt_tree* tree,
               const float* target_logits, const int32_t* target_argmax, const float* draft_q, const uint32_t* u_accept,
               const uint32_t* u_final, int stride, int32_t* accept_len, int32_t* path_idx, int32_t* out_tokens,
               int32_t* n_out) {
    if (!ctx || B < 1 || !tree || !tree->token || !tree->parent || tree->n < 1 || tree->n > TLT_MAX_TREE || stride < 1 ||
        !accept_len || !path_idx || !out_tokens || !n_out)
        return TLT_EINVAL;
    if (B > ctx->max_batch || tree->n > ctx->max_n) return TLT_ESHAPE;
    hipStream_t s = (hipStream_t)stream;
    const int n = tree->n, V = ctx->cfg.vocab;
    if (mode == 0) {
        if (!target_argmax && !target_logits) return TLT_EINVAL;
        const int32_t* am = target_argmax;
        if (!am) {
            int32_t* tmp = (int32_t*)(ctx->ws + ctx->plan.argmax);
            TLT_RUN(ctx, s, CLS_OTHER, 0, (double)B * n * V * 4, row_argmax(s, B * n, V, target_logits, tmp));
            am = tmp;
        }
        TLT_RUN(ctx, s, CLS_OTHER, 0, 0,
                accept_greedy(s, B, n, V, stride, tree->token, tree->parent, target_logits, am, accept_len, path_idx,
                              out_tokens, n_out));
        return TLT_OK;
    }
    if (mode == 1) {
        if (!target_logits || !draft_q || !u_accept || !u_final || !(temperature > 0.f)) return TLT_EINVAL;
        int rc = ensure_status(ctx, s);
        if (rc) return rc;
        TLT_RUN(ctx, s, CLS_OTHER, 0, 0,
                accept_sample(s, B, n, V, stride, temperature, tree->token, tree->parent, target_logits, draft_q, u_accept,
                              u_final, accept_len, path_idx, out_tokens, n_out, ctx->ws + ctx->plan.accept_ws,
                              status_word(ctx)));
        return TLT_OK;
    }
    if (mode == 2) {
        if (!target_logits || !u_accept || !u_final || !(temperature > 0.f)) return TLT_EINVAL;
        TLT_RUN(ctx, s, CLS_OTHER, 0, 0,
                accept_target_only(s, B, n, V, stride, temperature, tree->token, tree->parent, target_logits, u_accept,
                                   u_final, accept_len, path_idx, out_tokens, n_out));
        return TLT_OK;
    }
    return TLT_EINVAL;
}

// ---- sampling acceptance on the library's own static scratch (for callers that cannot allocate)
namespace {
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
constexpr int kMaxDevices = 64;
}  // namespace
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
namespace {
void* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each GPU (every GPU holds its own copy)

// The array's name is a host-side stand-in, not a device address: the address is asked for once per
// device, with that device current, and only that pointer is handed to kernels.
hipError_t static_scratch(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}
}  // namespace

int tlt_accept_sample_static(void* stream, int B, int vocab, float temperature, const tlt_tree* tree,
                             const float* target_logits, const float* draft_q, const uint32_t* u_accept,
                             const uint32_t* u_final, int stride, int32_t* accept_len, int32_t* path_idx,
                             int32_t* out_tokens, int32_t* n_out, uint32_t* status) {
    if (B < 1 || vocab < 1 || !tree || !tree->token || !tree->parent || tree->n < 1 || tree->n > TLT_MAX_TREE || stride < 1 ||
        !accept_len || !path_idx || !out_tokens || !n_out || !target_logits || !draft_q || !u_accept || !u_final ||
        !(temperature > 0.f))
        return TLT_EINVAL;
    // weights and rendezvous area, then one status word of the library's own (used when the caller passes none)
    const size_t need = accept_sample_workspace_bytes(B, vocab);
    if (need + 256 > kStaticScratchBytes) return TLT_ESHAPE;
    void* ptr = nullptr;
    if (static_scratch(&ptr) != hipSuccess) return TLT_EHIP;
    hipStream_t s = (hipStream_t)stream;
    unsigned int* st = status;
    if (!st) {
        st = (unsigned int*)((char*)ptr + kStaticScratchBytes - 256);
        if (zero_f32(s, 64, (float*)st) != hipSuccess) return TLT_EHIP;
    }
    hipError_t e = accept_sample(s, B, tree->n, vocab, stride, temperature, tree->token, tree->parent, target_logits, draft_q,
                                 u_accept, u_final, accept_len, path_idx, out_tokens, n_out, ptr, st);
    return e == hipSuccess ? TLT_OK : TLT_EHIP;
}

int tlt_kv_commit(tlt_ctx* ctx, void* stream, int B, tlt_kv* kv, const int32_t* accept_len, const int32_t* path_idx,
                  int stride) {
    if (!ctx || B < 1 || !accept_len || !path_idx || stride < 1) return TLT_EINVAL;
    if (!kv || !kv->k_pool || !kv->v_pool || !kv->block_table || !kv->seq_len || kv->n_pages < 1 || kv->max_pages < 1)
        return TLT_EINVAL;
    if (B > ctx->max_batch) return TLT_ESHAPE;
    hipStream_t s = (hipStream_t)stream;
    const tlt_model_cfg& c = ctx->cfg;
    // algorithmic bytes are data dependent (accept lengths live on the device): callers that want
    // a bandwidth figure compute 2 * sum(accept_len) * kv_bytes_per_token themselves
    TLT_RUN(ctx, s, CLS_COMMIT, 0, 0,
            kv_commit(s, c.dtype, B, c.n_layers, kv->k_pool, kv->v_pool, kv->n_pages, kv->block_table, kv->seq_len,
                      kv->max_pages, c.page_size, c.n_kv_heads, c.head_dim, accept_len, path_idx, stride));
    return TLT_OK;
}

size_t tlt_attention_workspace_bytes(int B, int n, int n_q_heads, int n_kv_heads, int head_dim, int max_ctx) {
    if (B < 1 || n < 1 || n > TLT_MAX_TREE || n_q_heads < 1 || n_kv_heads < 1 || n_q_heads % n_kv_heads || max_ctx < 1) return 0;
    return attention_workspace_bytes(B, n, n_q_heads, n_kv_heads, head_dim, max_ctx);
}

int tlt_attention(void* stream, int dtype, int B, int n, int n_q_heads, int n_kv_heads, int head_dim, int page_size,
                  const void* qkv, const uint64_t* anc_mask, const tlt_kv* kv, void* out, void* ws, size_t ws_bytes, int impl) {
    if (B < 1 || n < 1 || n > TLT_MAX_TREE || n_q_heads < 1 || n_kv_heads < 1 || n_q_heads % n_kv_heads || head_dim < 64 ||
        head_dim % 64 || head_dim > 256 || page_size < 1 || (dtype != TLT_F32 && dtype != TLT_BF16) || !qkv || !anc_mask || !out ||
        !ws)
        return TLT_EINVAL;
    if (!kv || !kv->k_pool || !kv->v_pool || !kv->block_table || !kv->seq_len || kv->n_pages < 1 || kv->max_pages < 1 ||
        kv->seq_len_bound < 0)
        return TLT_EINVAL;
    if ((int64_t)kv->seq_len_bound + n > (int64_t)kv->max_pages * page_size) return TLT_ENOPAGES;
    Rows rows;
    rows.B = B;
    rows.n = n;
    rows.mask = anc_mask;
    rows.mask_words = 1;
    rows.n_region = n;
    KVLayer k;
    k.k = kv->k_pool;
    k.v = kv->v_pool;
    k.n_pages = kv->n_pages;
    k.block_table = kv->block_table;
    k.seq_len = kv->seq_len;
    k.max_pages = kv->max_pages;
    k.page_size = page_size;
    k.n_kv = n_kv_heads;
    k.d = head_dim;
    k.seq_len_bound = kv->seq_len_bound;
    hipError_t e = attention((hipStream_t)stream, dtype, rows, k, qkv, out, n_q_heads, ws, ws_bytes, impl);
    return e == hipSuccess ? TLT_OK : (e == hipErrorInvalidValue ? TLT_ESHAPE : TLT_EHIP);
}

int tlt_gemm_glu(void* stream, int M, int N, int K, const void* A, const void* Wg, const void* Wu, void* act) {
    if (M < 1 || N < 1 || K < 1 || !A || !Wg || !Wu || !act) return TLT_EINVAL;
    if (!gemm_glu_supported(TLT_BF16, M, N, K, A, Wg, Wu) || ((uintptr_t)act & 7) != 0) return TLT_ENOTIMPL;   // (8-byte stores)
    return gemm_glu((hipStream_t)stream, M, N, K, A, Wg, Wu, act) == hipSuccess ? TLT_OK : TLT_EHIP;
}

int tlt_gemm_argmax(void* stream, int M, int N, int K, const void* A, const void* W, void* ws, size_t ws_bytes,
                    int32_t* out) {
    if (M < 1 || N < 1 || K < 1 || !A || !W || !ws || !out) return TLT_EINVAL;
    if (!gemm_argmax_supported(TLT_BF16, M, N, K, A, W)) return TLT_ENOTIMPL;
    if (ws_bytes < gemm_argmax_workspace_bytes(M, N)) return TLT_ESHAPE;
    return gemm_argmax((hipStream_t)stream, M, N, K, A, W, ws, out) == hipSuccess ? TLT_OK : TLT_EHIP;
}

int tlt_gemm(void* stream, int dtype, int out_mode, int M, int N, int K, const void* A, const void* W, void* C) {
    if (M < 0 || N < 1 || K < 1 || !A || !W || !C || (dtype != TLT_F32 && dtype != TLT_BF16) || out_mode < 0 || out_mode > 2)
        return TLT_EINVAL;
    return gemm((hipStream_t)stream, dtype, out_mode, M, N, K, A, W, C) == hipSuccess ? TLT_OK : TLT_EHIP;
}

int tlt_mfma_stream(void* stream, const void* frags, float* out, int iters) {
    if (!frags || !out || iters < 1 || iters > (1 << 20) || ((uintptr_t)frags & 15) != 0) return TLT_EINVAL;
    return mfma_stream((hipStream_t)stream, frags, out, iters) == hipSuccess ? TLT_OK : TLT_EHIP;
}

int tlt_profile_begin(tlt_ctx* ctx, int enable) {
    if (!ctx) return TLT_EINVAL;
    ctx->prof_on = enable != 0;
    if (enable == 1) ctx->recs.clear();
    return TLT_OK;
}

int tlt_profile_read(tlt_ctx* ctx, double* ms, int64_t* launches, double* flops, double* bytes) {
    if (!ctx || !ms || !launches || !flops || !bytes) return TLT_EINVAL;
    for (int i = 0; i < CLS_N; ++i) {
        ms[i] = 0;
        launches[i] = 0;
        flops[i] = 0;
        bytes[i] = 0;
    }
    for (size_t r = 0; r < ctx->recs.size(); ++r) {
        hipError_t e = hipEventSynchronize(ctx->events[2 * r + 1]);
        if (e != hipSuccess) return fail(ctx, e);
        float t = 0.f;
        e = hipEventElapsedTime(&t, ctx->events[2 * r], ctx->events[2 * r + 1]);
        if (e != hipSuccess) return fail(ctx, e);
        const ProfRec& rec = ctx->recs[r];
        ms[rec.cls] += t;
        launches[rec.cls] += 1;
        flops[rec.cls] += rec.flops;
        bytes[rec.cls] += rec.bytes;
    }
    ctx->recs.clear();
    return TLT_OK;
}


// ---- HIP-graph pool: the greedy step captured per batch bucket, drafter and target apart ------------------
struct tlt_graph_pool {
    tlt_ctx* ctx = nullptr;
    std::vector<int> buckets;
    int bound = 0;                 // sequence-length bound frozen into every graph
    hipStream_t cap = nullptr;     // capture stream (default priority)
    std::map<std::vector<uint64_t>, hipGraphExec_t> draft, target;
    char* snap = nullptr;          // device space for what a warm-up run must not change
    size_t snap_bytes = 0;
};

namespace {

struct Piece {
    void* p;
    size_t bytes;
};

// fn runs once for real on the pool's stream (first-use set-up such as kernel attributes must not fall into a
// capture), the buffers in `keep` get their contents back, and then fn is captured and instantiated.
int capture_graph(tlt_graph_pool* g, const std::vector<Piece>& keep, const std::function<int(hipStream_t)>& fn,
                  hipGraphExec_t* out) {
    tlt_ctx* ctx = g->ctx;
    size_t total = 0;
    for (const Piece& k : keep) total += (k.bytes + 255) & ~(size_t)255;
    hipError_t e;
    if (total > g->snap_bytes) {
        if (g->snap) (void)hipFree(g->snap);
        g->snap = nullptr;
        g->snap_bytes = 0;
        if ((e = hipMalloc((void**)&g->snap, total)) != hipSuccess) return fail(ctx, e);
        g->snap_bytes = total;
    }
    size_t off = 0;
    for (const Piece& k : keep) {
        if ((e = hipMemcpyAsync(g->snap + off, k.p, k.bytes, hipMemcpyDeviceToDevice, g->cap)) != hipSuccess) return fail(ctx, e);
        off += (k.bytes + 255) & ~(size_t)255;
    }
    const bool prof = ctx->prof_on;   // events may not be recorded into a capture
    ctx->prof_on = false;
    int rc = fn(g->cap);
    if (rc == TLT_OK) {
        off = 0;
        for (const Piece& k : keep) {
            if ((e = hipMemcpyAsync(k.p, g->snap + off, k.bytes, hipMemcpyDeviceToDevice, g->cap)) != hipSuccess) rc = fail(ctx, e);
            off += (k.bytes + 255) & ~(size_t)255;
        }
    }
    if (rc == TLT_OK && (e = hipStreamSynchronize(g->cap)) != hipSuccess) rc = fail(ctx, e);
    if (rc == TLT_OK) {
        hipGraph_t graph = nullptr;
        if ((e = hipStreamBeginCapture(g->cap, hipStreamCaptureModeThreadLocal)) != hipSuccess) {
            rc = fail(ctx, e);
        } else {
            rc = fn(g->cap);
            e = hipStreamEndCapture(g->cap, &graph);   // always ends the capture, also after a failed call
            if (rc == TLT_OK && e != hipSuccess) rc = fail(ctx, e);
            if (rc == TLT_OK && (e = hipGraphInstantiate(out, graph, nullptr, nullptr, 0)) != hipSuccess) rc = fail(ctx, e);
            if (graph) (void)hipGraphDestroy(graph);
        }
    }
    ctx->prof_on = prof;
    return rc;
}

void key_kv(std::vector<uint64_t>& k, const tlt_kv* kv) {
    k.push_back((uint64_t)(uintptr_t)kv->k_pool);
    k.push_back((uint64_t)(uintptr_t)kv->v_pool);
    k.push_back((uint64_t)kv->n_pages);
    k.push_back((uint64_t)(uintptr_t)kv->block_table);
    k.push_back((uint64_t)(uintptr_t)kv->seq_len);
    k.push_back((uint64_t)kv->max_pages);
}

void key_tree(std::vector<uint64_t>& k, const tlt_tree* t) {
    k.push_back((uint64_t)(uintptr_t)t->token);
    k.push_back((uint64_t)(uintptr_t)t->parent);
    k.push_back((uint64_t)(uintptr_t)t->depth);
    k.push_back((uint64_t)(uintptr_t)t->anc_mask);
    k.push_back((uint64_t)(uintptr_t)t->score);
    k.push_back((uint64_t)t->n);
}

}  // namespace

int tlt_graph_pool_create(tlt_ctx* ctx, const int32_t* buckets, int n_buckets, int seq_len_bound, tlt_graph_pool** out) {
    if (!ctx || !out || !buckets || n_buckets < 1 || seq_len_bound < 0) return TLT_EINVAL;
    for (int i = 0; i < n_buckets; ++i)
        if (buckets[i] < 1 || buckets[i] > ctx->max_batch || (i > 0 && buckets[i] <= buckets[i - 1])) return TLT_EINVAL;
    tlt_graph_pool* g = new (std::nothrow) tlt_graph_pool();
    if (!g) return TLT_EINVAL;
    g->ctx = ctx;
    g->buckets.assign(buckets, buckets + n_buckets);
    g->bound = seq_len_bound;
    hipError_t e = hipStreamCreateWithFlags(&g->cap, hipStreamNonBlocking);
    if (e != hipSuccess) {
        delete g;
        return fail(ctx, e);
    }
    *out = g;
    return TLT_OK;
}

int tlt_graph_pool_destroy(tlt_graph_pool* g) {
    if (!g) return TLT_OK;
    for (auto& kv : g->draft) (void)hipGraphExecDestroy(kv.second);
    for (auto& kv : g->target) (void)hipGraphExecDestroy(kv.second);
    if (g->snap) (void)hipFree(g->snap);
    if (g->cap) (void)hipStreamDestroy(g->cap);
    delete g;
    return TLT_OK;
}

int tlt_graph_pool_count(const tlt_graph_pool* g, int32_t* n_draft, int32_t* n_target) {
    if (!g || !n_draft || !n_target) return TLT_EINVAL;
    *n_draft = (int32_t)g->draft.size();
    *n_target = (int32_t)g->target.size();
    return TLT_OK;
}

int tlt_graph_pool_step(tlt_graph_pool* g, void* stream, int B, int depth, int topk, int n_verify, const tlt_step_args* a) {
    if (!g || !a || !a->draft_kv || !a->kv || !a->tree || B < 1) return TLT_EINVAL;
    if (!a->new_tokens || !a->new_src || !a->n_new || !a->hidden || !a->argmax || !a->hidden_out || !a->accept_len ||
        !a->path_idx || !a->out_tokens || !a->n_out || a->stride < 1 || a->new_stride < 1 || a->hidden_n < 1)
        return TLT_EINVAL;
    tlt_ctx* ctx = g->ctx;
    int Bk = 0;
    for (int b : g->buckets)
        if (b >= B) {
            Bk = b;
            break;
        }
    if (Bk == 0) return TLT_ESHAPE;
    hipStream_t s = (hipStream_t)stream;
    tlt_kv dkv = *a->draft_kv, kv = *a->kv;
    dkv.seq_len_bound = kv.seq_len_bound = g->bound;
    tlt_tree tree = *a->tree;
    const int h = ctx->cfg.hidden;

    std::vector<uint64_t> dkey = {(uint64_t)Bk, (uint64_t)depth, (uint64_t)topk, (uint64_t)n_verify,
                                  (uint64_t)(uintptr_t)a->new_tokens, (uint64_t)(uintptr_t)a->new_src,
                                  (uint64_t)(uintptr_t)a->n_new, (uint64_t)a->new_stride,
                                  (uint64_t)(uintptr_t)a->hidden, (uint64_t)a->hidden_n};
    key_kv(dkey, &dkv);
    key_tree(dkey, &tree);
    std::vector<uint64_t> tkey = {(uint64_t)Bk, (uint64_t)(uintptr_t)a->argmax, (uint64_t)(uintptr_t)a->hidden_out,
                                  (uint64_t)a->stride, (uint64_t)(uintptr_t)a->accept_len, (uint64_t)(uintptr_t)a->path_idx,
                                  (uint64_t)(uintptr_t)a->out_tokens, (uint64_t)(uintptr_t)a->n_out};
    key_kv(tkey, &kv);
    key_tree(tkey, &tree);

    const bool need_draft = g->draft.find(dkey) == g->draft.end();
    const bool need_target = g->target.find(tkey) == g->target.end();
    if (need_draft || need_target) {
        // captures are rare: everything the caller has queued ends first, so the warm-up runs see its state
        hipError_t e = hipStreamSynchronize(s);
        if (e != hipSuccess) return fail(ctx, e);
    }
    if (need_draft) {
        std::vector<Piece> keep = {{dkv.seq_len, (size_t)Bk * 4}};
        hipGraphExec_t exec = nullptr;
        int rc = capture_graph(g, keep, [&](hipStream_t cs) {
            return tlt_draft_expand(ctx, cs, Bk, depth, topk, n_verify, 0, a->new_tokens, a->new_src, a->n_new, a->new_stride,
                                    a->hidden, a->hidden_n, nullptr, &dkv, &tree);
        }, &exec);
        if (rc != TLT_OK) return rc;
        g->draft[dkey] = exec;
    }
    if (need_target) {
        const size_t row = (size_t)Bk * a->stride * 4;
        std::vector<Piece> keep = {{kv.seq_len, (size_t)Bk * 4}, {a->accept_len, (size_t)Bk * 4}, {a->n_out, (size_t)Bk * 4},
                                   {a->path_idx, row}, {a->out_tokens, row},
                                   {(void*)a->hidden, (size_t)Bk * a->hidden_n * h * 4}};   // hidden_out may be the same buffer
        hipGraphExec_t exec = nullptr;
        int rc = capture_graph(g, keep, [&](hipStream_t cs) {
            int r = tlt_verify_forward(ctx, cs, Bk, &tree, &kv, nullptr, a->argmax, nullptr, a->hidden_out);
            if (r == TLT_OK)
                r = tlt_accept(ctx, cs, Bk, 0, 1.0f, &tree, nullptr, a->argmax, nullptr, nullptr, nullptr, a->stride, a->accept_len,
                               a->path_idx, a->out_tokens, a->n_out);
            if (r == TLT_OK) r = tlt_kv_commit(ctx, cs, Bk, &kv, a->accept_len, a->path_idx, a->stride);
            return r;
        }, &exec);
        if (rc != TLT_OK) return rc;
        g->target[tkey] = exec;
    }
    hipError_t e = hipGraphLaunch(g->draft[dkey], s);
    if (e == hipSuccess) e = hipGraphLaunch(g->target[tkey], s);
    return e == hipSuccess ? TLT_OK : fail(ctx, e);
}

}  // extern "C"
