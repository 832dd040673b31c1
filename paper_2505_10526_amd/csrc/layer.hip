// verify_layer and lm_head_logits: the parallel forward of the verify step
// (paper Section 2.1: the target scores all drafted positions in a single forward pass) as a fixed sequence of kernel
// launches on the caller's stream.
#include "kernels.h"

namespace massv {

struct LayerLayout { size_t xn, qkv, qrot, attn, h, gu, proj, h32, partial, attn_ws, total; };

// The four projections of a layer as launch_gemm sees them (pointers filled in by the caller).
struct LayerGemms { GemmArgs qkv, op, gu, dn; };

static LayerGemms layer_gemms(const massv_layer_desc& d) {
    const massv_attn_desc& a = d.attn;
    const int M = a.batch * a.n_query, H = d.hidden, F = d.mlp;
    const int nq = a.n_q_heads * a.head_dim, nkv = a.n_kv_heads * a.head_dim;
    const bool bf = a.dtype == MASSV_BF16;
    LayerGemms g = {};
    g.qkv.n[0] = nq; g.qkv.n[1] = nkv; g.qkv.n[2] = nkv; g.qkv.M = M; g.qkv.K = H;
    g.qkv.epilogue = bf ? EPI_PARTIAL : EPI_STORE; g.qkv.kid = MASSV_K_QKV;
    g.op.n[0] = H; g.op.M = M; g.op.K = nq; g.op.epilogue = bf ? EPI_PARTIAL : EPI_RESIDUAL; g.op.kid = MASSV_K_OPROJ;
    g.gu.n[0] = F; g.gu.n[1] = F; g.gu.M = M; g.gu.K = H; g.gu.epilogue = EPI_GATED; g.gu.kid = MASSV_K_GATEUP;
    g.dn.n[0] = H; g.dn.M = M; g.dn.K = F; g.dn.epilogue = bf ? EPI_PARTIAL : EPI_RESIDUAL; g.dn.kid = MASSV_K_DOWN;
    GemmArgs* all[4] = {&g.qkv, &g.op, &g.gu, &g.dn};
    for (GemmArgs* p : all) { p->act = d.act; p->dtype = a.dtype; }
    return g;
}

static LayerLayout layer_layout(const massv_layer_desc& d) {
    const massv_attn_desc& a = d.attn;
    const size_t es = a.dtype == MASSV_F32 ? 4 : 2;
    const size_t M = (size_t)a.batch * a.n_query;
    const size_t nq = (size_t)a.n_q_heads * a.head_dim, nkv = (size_t)a.n_kv_heads * a.head_dim;
    const bool bf = a.dtype == MASSV_BF16;          // bf16 activations that feed a projection are kept in operand order
    const size_t Mp = bf ? (M + 15) / 16 * 16 : M;
    const LayerGemms g = layer_gemms(d);
    size_t part = gemm_partial_bytes(g.qkv);
    if (gemm_partial_bytes(g.op) > part) part = gemm_partial_bytes(g.op);
    if (gemm_partial_bytes(g.dn) > part) part = gemm_partial_bytes(g.dn);
    LayerLayout l;
    size_t o = 0;
    l.xn = o;   o = align_up(o + Mp * d.hidden * es, 256);
    l.qkv = o;  o = align_up(o + (bf ? 0 : M * (nq + 2 * nkv) * es), 256);
    l.qrot = o; o = align_up(o + M * nq * es, 256);
    l.attn = o; o = align_up(o + Mp * nq * es, 256);
    l.h = o;    o = align_up(o + Mp * d.mlp * es, 256);
    l.gu = o;   o = align_up(o + (bf ? 0 : M * 2 * d.mlp * 4), 256);
    l.proj = o; o = align_up(o + (bf ? 0 : M * d.hidden * 4), 256);   // fp32: a block's output ahead of its output norm
    l.h32 = o;  o = align_up(o + (bf ? M * d.hidden * 4 : 0), 256);   // bf16: the stream between the two blocks, fp32
    l.partial = o; o = align_up(o + part, 256);
    l.attn_ws = o; o = align_up(o + attention_workspace(a), 256);
    l.total = o;
    return l;
}

static int check_layer_desc(const massv_layer_desc* d) {
    if (!d) return MASSV_EINVAL;
    const int rc = check_attn_desc(&d->attn);
    if (rc != MASSV_OK) return rc;
    if (d->hidden < 1 || d->mlp < 1) return MASSV_EINVAL;
    if (d->act != MASSV_ACT_SILU && d->act != MASSV_ACT_GELU_TANH) return MASSV_EINVAL;
    if (!(d->norm_eps >= 0.f) || !(d->rope_theta > 0.f)) return MASSV_EINVAL;
    if (d->attn.dtype == MASSV_BF16) {
        const int M = d->attn.batch * d->attn.n_query;
        if (M > MASSV_MAX_ROWS) return MASSV_EUNSUPPORTED;
        if (d->hidden % 32 || d->mlp % 32 || (d->attn.n_q_heads * d->attn.head_dim) % 32) return MASSV_EUNSUPPORTED;
        if (d->hidden > 8192) return MASSV_EUNSUPPORTED;
    }
    return MASSV_OK;
}

}  // namespace massv

using namespace massv;

extern "C" size_t massv_verify_layer_workspace(const massv_layer_desc* desc) {
    if (check_layer_desc(desc) != MASSV_OK) return 0;
    return layer_layout(*desc).total;
}

static int check_layer_weights(const massv_layer_desc* desc, const massv_layer_weights* w) {
    if (!w) return MASSV_EINVAL;
    if (!w->ln1 || !w->wq || !w->wk || !w->wv || !w->wo || !w->ln2 || !w->wg || !w->wu || !w->wd) return MASSV_EINVAL;
    if (desc->qkv_bias && (!w->bq || !w->bk || !w->bv)) return MASSV_EINVAL;
    return MASSV_OK;
}

// One layer.  xn_ready: the workspace already holds rmsnorm(x, ln1) in operand order (written by the
// previous layer's last kernel); next_ln: gains of the norm that follows this layer (the next layer's
// ln1), fused into this layer's last kernel when not NULL.  Both are bf16-path options.
static int run_layer(const massv_layer_desc* desc, const massv_layer_weights* w, void* x, const int32_t* pos,
                     void* k_cache, void* v_cache, const int32_t* kv_len, void* workspace,
                     const LayerLayout& lay, bool xn_ready, const void* next_ln, hipStream_t st) {
    int rc;
    const massv_attn_desc& a = desc->attn;
    char* ws = (char*)workspace;
    const int M = a.batch * a.n_query, H = desc->hidden;
    const bool bias = desc->qkv_bias != 0;
    const bool bf = a.dtype == MASSV_BF16;
    const size_t Mp = (size_t)(M + 15) / 16 * 16;
    float* partial = (float*)(ws + lay.partial);

    LayerGemms g = layer_gemms(*desc);
    g.qkv.x = ws + lay.xn;
    g.qkv.w[0] = w->wq; g.qkv.w[1] = w->wk; g.qkv.w[2] = w->wv;
    if (!bf) { g.qkv.bias[0] = bias ? w->bq : nullptr; g.qkv.bias[1] = bias ? w->bk : nullptr; g.qkv.bias[2] = bias ? w->bv : nullptr; }
    g.qkv.y = bf ? (void*)partial : (void*)(ws + lay.qkv);
    g.op.x = ws + lay.attn; g.op.w[0] = w->wo; g.op.residual = x; g.op.y = bf ? (void*)partial : x;
    if (!bf && w->post_attn_norm) { g.op.epilogue = EPI_STORE; g.op.residual = nullptr; g.op.y = ws + lay.proj; }
    g.gu.x = ws + lay.xn; g.gu.w[0] = w->wg; g.gu.w[1] = w->wu; g.gu.y = ws + lay.h; g.gu.scratch = ws + lay.gu;
    g.dn.x = ws + lay.h; g.dn.w[0] = w->wd; g.dn.residual = x; g.dn.y = bf ? (void*)partial : x;
    if (!bf && w->post_mlp_norm) { g.dn.epilogue = EPI_STORE; g.dn.residual = nullptr; g.dn.y = ws + lay.proj; }

    // shape checks for every projection before the first launch
    if ((rc = gemm_supported(g.qkv)) != MASSV_OK) return rc;
    if ((rc = gemm_supported(g.op)) != MASSV_OK) return rc;
    if ((rc = gemm_supported(g.gu)) != MASSV_OK) return rc;
    if ((rc = gemm_supported(g.dn)) != MASSV_OK) return rc;

    if (!bf) {
        if ((rc = launch_rmsnorm(x, w->ln1, ws + lay.xn, M, H, desc->norm_eps, st)) != MASSV_OK) return rc;
        if ((rc = launch_gemm(g.qkv, st)) != MASSV_OK) return rc;
        if ((rc = launch_rope_append(ws + lay.qkv, pos, kv_len, ws + lay.qrot, k_cache, v_cache, w->q_norm, w->k_norm,
                                     desc->norm_eps, a, desc->rope_theta, st)) != MASSV_OK) return rc;
        if ((rc = launch_attention(a, ws + lay.qrot, k_cache, v_cache, kv_len, ws + lay.attn, ws + lay.attn_ws, false, st)) != MASSV_OK) return rc;
        if ((rc = launch_gemm(g.op, st)) != MASSV_OK) return rc;
        if (w->post_attn_norm &&
            (rc = launch_postnorm_residual(x, ws + lay.proj, w->post_attn_norm, M, H, desc->norm_eps, st)) != MASSV_OK) return rc;
        if ((rc = launch_rmsnorm(x, w->ln2, ws + lay.xn, M, H, desc->norm_eps, st)) != MASSV_OK) return rc;
        if ((rc = launch_gemm(g.gu, st)) != MASSV_OK) return rc;
        if ((rc = launch_gemm(g.dn, st)) != MASSV_OK) return rc;
        if (w->post_mlp_norm) return launch_postnorm_residual(x, ws + lay.proj, w->post_mlp_norm, M, H, desc->norm_eps, st);
        return MASSV_OK;
    }
    // bf16: the narrow projections leave fp32 partial sums per K slab; the row-wise kernel that has to
    // run next anyway (rotary + append, residual + norm) sums them.
    const size_t wq = (size_t)(a.n_q_heads + 2 * a.n_kv_heads) * a.head_dim;
    if (!xn_ready && (rc = launch_rmsnorm_packed(x, w->ln1, ws + lay.xn, M, H, desc->norm_eps, st)) != MASSV_OK) return rc;
    if ((rc = launch_gemm(g.qkv, st)) != MASSV_OK) return rc;
    if ((rc = launch_qkv_finish(partial, gemm_plan(g.qkv).slabs, Mp * wq, bias ? w->bq : nullptr, bias ? w->bk : nullptr,
                                bias ? w->bv : nullptr, pos, kv_len, ws + lay.qrot, k_cache, v_cache, w->q_norm, w->k_norm,
                                desc->norm_eps, a, desc->rope_theta, st)) != MASSV_OK) return rc;
    if ((rc = launch_attention(a, ws + lay.qrot, k_cache, v_cache, kv_len, ws + lay.attn, ws + lay.attn_ws, true, st)) != MASSV_OK) return rc;
    if ((rc = launch_gemm(g.op, st)) != MASSV_OK) return rc;
    float* h32 = (float*)(ws + lay.h32);
    if ((rc = launch_residual_finish(partial, gemm_plan(g.op).slabs, Mp * H, x, nullptr, h32, w->post_attn_norm, w->ln2,
                                     ws + lay.xn, M, H, desc->norm_eps, st)) != MASSV_OK) return rc;
    if ((rc = launch_gemm(g.gu, st)) != MASSV_OK) return rc;
    if ((rc = launch_gemm(g.dn, st)) != MASSV_OK) return rc;
    return launch_residual_finish(partial, gemm_plan(g.dn).slabs, Mp * H, x, h32, nullptr, w->post_mlp_norm, next_ln,
                                  next_ln ? ws + lay.xn : nullptr, M, H, desc->norm_eps, st);
}

extern "C" int massv_verify_layer(const massv_layer_desc* desc, const massv_layer_weights* w,
                                  void* x, const int32_t* pos, void* k_cache, void* v_cache,
                                  const int32_t* kv_len, void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_layer_desc(desc);
    if (rc != MASSV_OK) return rc;
    if (!x || !pos || !k_cache || !v_cache || !kv_len) return MASSV_EINVAL;
    if ((rc = check_layer_weights(desc, w)) != MASSV_OK) return rc;
    const LayerLayout lay = layer_layout(*desc);
    if (!workspace || workspace_bytes < lay.total) return MASSV_EWORKSPACE;
    return run_layer(desc, w, x, pos, k_cache, v_cache, kv_len, workspace, lay, false, nullptr, (hipStream_t)stream);
}

extern "C" int massv_verify_layers(const massv_layer_desc* desc, const massv_layer_weights* weights, int32_t n_layers,
                                   void* x, const int32_t* pos, void* const* k_caches, void* const* v_caches,
                                   const int32_t* kv_len, const int32_t* windows, const float* rope_thetas,
                                   void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_layer_desc(desc);
    if (rc != MASSV_OK) return rc;
    if (n_layers < 1 || !weights || !x || !pos || !k_caches || !v_caches || !kv_len) return MASSV_EINVAL;
    for (int l = 0; l < n_layers; ++l) {
        if ((rc = check_layer_weights(desc, weights + l)) != MASSV_OK) return rc;
        if (!k_caches[l] || !v_caches[l]) return MASSV_EINVAL;
        if (windows && windows[l] < 0) return MASSV_EINVAL;
        if (rope_thetas && !(rope_thetas[l] > 0.f)) return MASSV_EINVAL;
    }
    const LayerLayout lay = layer_layout(*desc);
    if (!workspace || workspace_bytes < lay.total) return MASSV_EWORKSPACE;
    const bool bf = desc->attn.dtype == MASSV_BF16;
    for (int l = 0; l < n_layers; ++l) {
        // bf16: the norm that opens layer l+1 is computed by the kernel that closes layer l
        const void* next_ln = (bf && l + 1 < n_layers) ? weights[l + 1].ln1 : nullptr;
        massv_layer_desc dl = *desc;                    // this layer's window and rotary base
        if (windows) dl.attn.window = windows[l];
        if (rope_thetas) dl.rope_theta = rope_thetas[l];
        rc = run_layer(&dl, weights + l, x, pos, k_caches[l], v_caches[l], kv_len, workspace, lay,
                       bf && l > 0, next_ln, (hipStream_t)stream);
        if (rc != MASSV_OK) return rc;
    }
    return MASSV_OK;
}

static int check_lm_head(int32_t M, int32_t H, int32_t V, int32_t dtype) {
    if (M < 1 || H < 1 || V < 1) return MASSV_EINVAL;
    if (dtype != MASSV_F32 && dtype != MASSV_BF16) return MASSV_EINVAL;
    if (dtype == MASSV_BF16 && (M > MASSV_MAX_ROWS || H % 32 || V % 16)) return MASSV_EUNSUPPORTED;
    return MASSV_OK;
}

extern "C" size_t massv_lm_head_logits_workspace(int32_t M, int32_t H, int32_t V, int32_t dtype) {
    if (check_lm_head(M, H, V, dtype) != MASSV_OK) return 0;
    return dtype == MASSV_F32 ? align_up((size_t)M * H * 4, 256) : align_up(packed_elems(M, H) * 2, 256);
}

extern "C" int massv_lm_head_logits(const void* x, const void* final_norm, const void* w_lm, float* logits,
                                    int32_t M, int32_t H, int32_t V, float norm_eps, int32_t dtype,
                                    void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_lm_head(M, H, V, dtype);
    if (rc != MASSV_OK) return rc;
    if (!x || !w_lm || !logits) return MASSV_EINVAL;
    if (!(norm_eps >= 0.f)) return MASSV_EINVAL;
    if (!workspace || workspace_bytes < massv_lm_head_logits_workspace(M, H, V, dtype)) return MASSV_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    GemmArgs g = {};
    g.x = x;
    if (dtype == MASSV_BF16) {                  // normalise (or only re-lay out) into operand order
        if ((rc = launch_rmsnorm_packed(x, final_norm, workspace, M, H, norm_eps, st)) != MASSV_OK) return rc;
        g.x = workspace;
    } else if (final_norm) {
        if ((rc = launch_rmsnorm(x, final_norm, workspace, M, H, norm_eps, st)) != MASSV_OK) return rc;
        g.x = workspace;
    }
    g.w[0] = w_lm; g.n[0] = V; g.y = logits; g.M = M; g.K = H;
    g.epilogue = EPI_LOGITS; g.dtype = dtype; g.kid = MASSV_K_LMHEAD;
    return launch_gemm(g, st);
}

// lm_head and the temperature-0 accept rule in one pass over the vocabulary projection: the projection's epilogue
// keeps, per row and workgroup, only the largest logit and its column, so the M x V logits are never written.
static GemmArgs greedy_gemm(int32_t M, int32_t H, int32_t V) {
    GemmArgs g = {};
    g.n[0] = V; g.M = M; g.K = H; g.epilogue = EPI_ARGMAX; g.dtype = MASSV_BF16; g.kid = MASSV_K_LMHEAD;
    return g;
}

static int check_greedy(int32_t B, int32_t gamma, int32_t H, int32_t V, int32_t dtype) {
    if (B < 1 || gamma < 0 || H < 1 || V < 1) return MASSV_EINVAL;
    if (dtype != MASSV_F32 && dtype != MASSV_BF16) return MASSV_EINVAL;
    if (dtype != MASSV_BF16) return MASSV_EUNSUPPORTED;
    if (gamma > 15 || (int64_t)B * (gamma + 1) > MASSV_MAX_ROWS || H % 32 || V % 16) return MASSV_EUNSUPPORTED;
    return MASSV_OK;
}

extern "C" size_t massv_lm_head_greedy_accept_workspace(int32_t B, int32_t gamma, int32_t H, int32_t V, int32_t dtype) {
    if (check_greedy(B, gamma, H, V, dtype) != MASSV_OK) return 0;
    const int M = B * (gamma + 1);
    const GemmPlan p = gemm_plan(greedy_gemm(M, H, V));
    return align_up(packed_elems(M, H) * 2, 256) + align_up((size_t)M * p.groups * sizeof(RowPartial), 256);
}

extern "C" int massv_lm_head_greedy_accept(const void* x, const void* final_norm, const void* w_lm,
                                           const int32_t* draft_tokens, int32_t B, int32_t gamma, int32_t H, int32_t V,
                                           float norm_eps, int32_t dtype, int32_t* n_accepted, int32_t* out_tokens,
                                           void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_greedy(B, gamma, H, V, dtype);
    if (rc != MASSV_OK) return rc;
    if (!x || !w_lm || !n_accepted || !out_tokens || (gamma > 0 && !draft_tokens)) return MASSV_EINVAL;
    if (!(norm_eps >= 0.f)) return MASSV_EINVAL;
    if (!workspace || workspace_bytes < massv_lm_head_greedy_accept_workspace(B, gamma, H, V, dtype)) return MASSV_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    const int M = B * (gamma + 1);
    if ((rc = launch_rmsnorm_packed(x, final_norm, workspace, M, H, norm_eps, st)) != MASSV_OK) return rc;
    GemmArgs g = greedy_gemm(M, H, V);
    RowPartial* part = (RowPartial*)((char*)workspace + align_up(packed_elems(M, H) * 2, 256));
    g.x = workspace; g.w[0] = w_lm; g.y = part;
    if ((rc = launch_gemm(g, st)) != MASSV_OK) return rc;
    return launch_accept_decide_greedy(part, gemm_plan(g).groups, draft_tokens, B, gamma, V, n_accepted, out_tokens, st);
}

// lm_head and the accept rule in one call at any temperature.  T = 0: the greedy path above (no logits written).
// T > 0: the projection writes the logits (the accept rule gathers p(x_i) from them and re-reads one row per sequence
// for the final draw) and its epilogue leaves, per row and workgroup, the largest logit, its column and the sum of
// exponentials -- the target half of the accept call's first pass, which then streams the draft rows only.
static GemmArgs stats_gemm(int32_t M, int32_t H, int32_t V, float temperature) {
    GemmArgs g = {};
    g.n[0] = V; g.M = M; g.K = H; g.epilogue = EPI_LOGITS_STATS; g.dtype = MASSV_BF16; g.kid = MASSV_K_LMHEAD;
    g.temperature = temperature;
    return g;
}

extern "C" size_t massv_lm_head_accept_workspace(int32_t B, int32_t gamma, int32_t H, int32_t V, int32_t dtype) {
    if (check_greedy(B, gamma, H, V, dtype) != MASSV_OK) return 0;
    const int M = B * (gamma + 1);
    const GemmPlan p = gemm_plan(stats_gemm(M, H, V, 1.f));
    const size_t sampled = align_up(packed_elems(M, H) * 2, 256) + align_up((size_t)M * p.groups * sizeof(RowPartial), 256) +
                           accept_prestats_bytes(B, gamma, V);
    const size_t greedy = massv_lm_head_greedy_accept_workspace(B, gamma, H, V, dtype);
    return sampled > greedy ? sampled : greedy;
}

extern "C" int massv_lm_head_accept(const void* x, const void* final_norm, const void* w_lm,
                                    const float* draft_logits, const int32_t* draft_tokens, const float* uniforms,
                                    float temperature, int32_t B, int32_t gamma, int32_t H, int32_t V,
                                    float norm_eps, int32_t dtype, float* logits, int32_t* n_accepted, int32_t* out_tokens,
                                    void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_greedy(B, gamma, H, V, dtype);
    if (rc != MASSV_OK) return rc;
    if (!(temperature >= 0.f) || isinf(temperature)) return MASSV_EINVAL;     // also catches NaN
    if (!workspace || workspace_bytes < massv_lm_head_accept_workspace(B, gamma, H, V, dtype)) return MASSV_EWORKSPACE;
    if (temperature == 0.f)
        return massv_lm_head_greedy_accept(x, final_norm, w_lm, draft_tokens, B, gamma, H, V, norm_eps, dtype, n_accepted,
                                           out_tokens, workspace, workspace_bytes, stream);
    if (!x || !w_lm || !logits || !uniforms || !n_accepted || !out_tokens) return MASSV_EINVAL;
    if (gamma > 0 && (!draft_tokens || !draft_logits)) return MASSV_EINVAL;
    if (!(norm_eps >= 0.f)) return MASSV_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    const int M = B * (gamma + 1);
    if ((rc = launch_rmsnorm_packed(x, final_norm, workspace, M, H, norm_eps, st)) != MASSV_OK) return rc;
    GemmArgs g = stats_gemm(M, H, V, temperature);
    char* ws = (char*)workspace;
    RowPartial* part = (RowPartial*)(ws + align_up(packed_elems(M, H) * 2, 256));
    const int groups = gemm_plan(g).groups;
    void* accept_ws = (char*)part + align_up((size_t)M * groups * sizeof(RowPartial), 256);
    g.x = workspace; g.w[0] = w_lm; g.y = logits; g.stats = part;
    if ((rc = launch_gemm(g, st)) != MASSV_OK) return rc;
    return launch_accept_prestats(logits, part, groups, draft_logits, draft_tokens, uniforms, temperature, B, gamma, V,
                                  n_accepted, out_tokens, accept_ws, st);
}
