// Host-side composition of one SDXL-shaped transformer stage block (the U-Net denoiser's attention
// stage is the second workload shape of the guidance-branch forward, Sec. 4.1 / Sec. 5 setup):
//   g = GroupNorm32(x);  a = g + SelfAttn(LN(g));  b = a + CrossAttn(LN(a), ctx);
//   out = x + b + W2 (u * GELUerf(gate)) + b2,  [u, gate] = LN(b) W1^T + b1
// Thirteen launches: GroupNorm, LN, fused QKV GEMM (head-major scatter), self-attention, out-projection
// (+ residual), LN, Q GEMM, K/V GEMM on the text context, cross-attention, out-projection (+ residual),
// LN, GEGLU GEMM, down-projection (+ both residuals).
#include "attention.h"
#include "gemm.h"

int hyb_launch_layernorm(const float* x, const float* shift, const float* scale, size_t mod_stride, void* out,
                         int batch, int tokens, int hidden, float eps, hyb_dtype out_dtype, bool affine, hipStream_t st);
int hyb_launch_groupnorm(const float* x, const float* gamma, const float* beta, float* out, int batch, int tokens,
                         int channels, int groups, float eps, void* scratch, hipStream_t st);
size_t hyb_groupnorm_scratch_bytes(int batch, int groups);

namespace {

struct SdxlLayout {
    size_t g, h, q, k, v, o, ck, cv, ff, gn, splitk, splitk_bytes, total;
};

SdxlLayout sdxl_layout(const hyb_sdxl_block_desc& d) {
    const size_t es = hyb_dtype_size(d.dtype);
    const size_t B = d.batch, T = d.tokens, C = d.channels, S = d.n_ctx;
    SdxlLayout L;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t o = off;
        off += hyb_align_up(bytes, 256);
        return o;
    };
    L.g = take(B * T * C * 4);          // residual stream after GroupNorm (fp32)
    L.h = take(B * T * C * es);         // LayerNorm output
    L.q = take(B * T * C * es);
    L.k = take(B * T * C * es);
    L.v = take(B * T * C * es);
    L.o = take(B * T * C * es);
    L.ck = take(B * S * C * es);        // context keys / values, head-major
    L.cv = take(B * S * C * es);
    L.ff = take(B * T * 4 * C * es);    // GEGLU output
    L.gn = take(hyb_groupnorm_scratch_bytes(d.batch, d.groups));
    // fp32 planes of the GEMMs' k split: up to 8 for the context K/V projection (few rows), 3 for the down-projection
    const size_t kv_planes = 8 * B * S * 2 * C * 4, ff2_planes = 3 * B * T * C * 4;
    L.splitk_bytes = kv_planes > ff2_planes ? kv_planes : ff2_planes;
    L.splitk = take(L.splitk_bytes);
    L.total = off;
    return L;
}

int check_desc(const char* who, const hyb_sdxl_block_desc* d) {
    HYB_CHECK_PTR(d);
    HYB_CHECK_DTYPE(d->dtype);
    HYB_REQUIRE(d->batch >= 0 && d->tokens >= 0 && d->n_ctx > 0 && d->ctx_dim > 0, HYB_ERR_SHAPE, "%s: bad sizes", who);
    HYB_REQUIRE(d->head_dim == 64, HYB_ERR_SHAPE, "%s: head_dim %d is not supported (only 64)", who, d->head_dim);
    HYB_REQUIRE(d->heads > 0 && d->channels == d->heads * 64, HYB_ERR_SHAPE, "%s: channels %d != heads %d * 64", who, d->channels, d->heads);
    HYB_REQUIRE(d->channels <= 2048, HYB_ERR_SHAPE, "%s: channels %d exceeds 2048", who, d->channels);
    HYB_REQUIRE(d->groups > 0 && d->channels % d->groups == 0, HYB_ERR_SHAPE, "%s: channels %d not divisible by groups %d", who, d->channels, d->groups);
    HYB_REQUIRE(d->batch <= 65535, HYB_ERR_SHAPE, "%s: batch exceeds 65535", who);
    return HYB_OK;
}

}  // namespace

extern "C" size_t hyb_sdxl_block_workspace_bytes(const hyb_sdxl_block_desc* desc) {
    if (check_desc("hyb_sdxl_block_workspace_bytes", desc) != HYB_OK) return 0;
    return sdxl_layout(*desc).total;
}

extern "C" int hyb_sdxl_block_forward(const hyb_sdxl_block_desc* desc, const hyb_sdxl_block_weights* w,
                                      const float* x_in, const void* ctx, float* x_out,
                                      void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_desc("hyb_sdxl_block_forward", desc);
    if (rc) return rc;
    HYB_CHECK_PTR(w);
    const hyb_sdxl_block_desc& d = *desc;
    const int B = d.batch, T = d.tokens, C = d.channels, S = d.n_ctx, M = B * T;
    if (M == 0) return HYB_OK;
    HYB_CHECK_PTR(x_in); HYB_CHECK_PTR(ctx); HYB_CHECK_PTR(x_out); HYB_CHECK_PTR(workspace);
    HYB_CHECK_ALIGN(x_in); HYB_CHECK_ALIGN(ctx); HYB_CHECK_ALIGN(x_out); HYB_CHECK_ALIGN(workspace);
    const void* ptrs[] = {w->gn_g, w->gn_b, w->ln1_g, w->ln1_b, w->ln2_g, w->ln2_b, w->ln3_g, w->ln3_b, w->w_qkv1, w->w_o1,
                          w->b_o1, w->w_q2, w->w_kv2, w->w_o2, w->b_o2, w->w_ff1, w->b_ff1, w->w_ff2, w->b_ff2};
    for (const void* p : ptrs) {
        HYB_REQUIRE(p != nullptr, HYB_ERR_NULL, "hyb_sdxl_block_forward: a weight pointer is NULL");
        HYB_REQUIRE(((uintptr_t)p & 15u) == 0, HYB_ERR_ALIGN, "hyb_sdxl_block_forward: a weight pointer is not 16-byte aligned");
    }
    const SdxlLayout L = sdxl_layout(d);
    HYB_REQUIRE(workspace_bytes >= L.total, HYB_ERR_WORKSPACE, "hyb_sdxl_block_forward: workspace of %zu bytes is smaller than the %zu required", workspace_bytes, L.total);

    hipStream_t st = (hipStream_t)stream;
    char* ws = static_cast<char*>(workspace);
    const hyb_dtype dt = d.dtype;
    float* g = reinterpret_cast<float*>(ws + L.g);
    void* h = ws + L.h;
    void* o = ws + L.o;
    auto one = [&](int m, int n, int k) {
        GemmGroup gg = {};
        gg.count = 1; gg.n = n; gg.k = k; gg.p[0].m = m;
        gg.splitk_ws = ws + L.splitk; gg.splitk_bytes = L.splitk_bytes;
        return gg;
    };
    constexpr float kQScale = 0.125f * 1.4426950408889634f;      // softmax scale 1 / sqrt(64) times log2(e)
    auto attn = [&](void* q, void* k, void* v, int n_kv) {
        AttnArgs a = {q, k, v, o, nullptr, T, B, d.heads, T, n_kv, 0.125f};
        a.prescaled = dt == HYB_BF16;      // the q projections below store q times scale x log2(e) in that case
        return hyb_launch_attention(a, dt, st);
    };

    // g = GroupNorm(x): the residual stream of the block
    if ((rc = hyb_launch_groupnorm(x_in, w->gn_g, w->gn_b, g, B, T, C, d.groups, d.gn_eps, ws + L.gn, st))) return rc;
    // self-attention: a = g + (softmax(q k^T / 8) v) Wo^T + bo   (in place on g)
    if ((rc = hyb_launch_layernorm(g, w->ln1_b, w->ln1_g, 0, h, B, T, C, d.ln_eps, dt, true, st))) return rc;
    {
        GemmGroup gg = one(M, 3 * C, C);
        GemmProblem& p = gg.p[0];
        p.a = h; p.w = w->w_qkv1; p.q = ws + L.q; p.k = ws + L.k; p.v = ws + L.v;
        p.tokens = T; p.tok_offset = 0; p.n_total = T; p.heads = d.heads;
        if (dt == HYB_BF16) p.q_scale = kQScale;
        if ((rc = hyb_launch_gemm(gg, dt, dt, EPI_QKV, st))) return rc;
    }
    if ((rc = attn(ws + L.q, ws + L.k, ws + L.v, T))) return rc;
    {
        GemmGroup gg = one(M, C, C);
        GemmProblem& p = gg.p[0];
        p.a = o; p.w = w->w_o1; p.bias = w->b_o1; p.out = g; p.res = g; p.rows_per_gate = 1;
        if ((rc = hyb_launch_gemm(gg, dt, HYB_F32, EPI_GATE_RES, st))) return rc;
    }
    // cross-attention to the text context: b = a + (softmax(q kc^T / 8) vc) Wo2^T + bo2
    if ((rc = hyb_launch_layernorm(g, w->ln2_b, w->ln2_g, 0, h, B, T, C, d.ln_eps, dt, true, st))) return rc;
    {
        GemmGroup gg = one(M, C, C);
        GemmProblem& p = gg.p[0];
        p.a = h; p.w = w->w_q2; p.q = ws + L.q;
        p.tokens = T; p.tok_offset = 0; p.n_total = T; p.heads = d.heads;
        if (dt == HYB_BF16) p.q_scale = kQScale;
        if ((rc = hyb_launch_gemm(gg, dt, dt, EPI_QKV, st))) return rc;
    }
    {
        GemmGroup gg = one(B * S, 2 * C, d.ctx_dim);
        GemmProblem& p = gg.p[0];
        p.a = ctx; p.w = w->w_kv2; p.q = ws + L.ck; p.k = ws + L.cv;
        p.tokens = S; p.tok_offset = 0; p.n_total = S; p.heads = d.heads;
        if ((rc = hyb_launch_gemm(gg, dt, dt, EPI_QKV, st))) return rc;
    }
    if ((rc = attn(ws + L.q, ws + L.ck, ws + L.cv, S))) return rc;
    {
        GemmGroup gg = one(M, C, C);
        GemmProblem& p = gg.p[0];
        p.a = o; p.w = w->w_o2; p.bias = w->b_o2; p.out = g; p.res = g; p.rows_per_gate = 1;
        if ((rc = hyb_launch_gemm(gg, dt, HYB_F32, EPI_GATE_RES, st))) return rc;
    }
    // GEGLU feed-forward and the outer residual: out = x + b + (u * GELUerf(gate)) W2^T + b2
    if ((rc = hyb_launch_layernorm(g, w->ln3_b, w->ln3_g, 0, h, B, T, C, d.ln_eps, dt, true, st))) return rc;
    {
        GemmGroup gg = one(M, 4 * C, C);
        GemmProblem& p = gg.p[0];
        p.a = h; p.w = w->w_ff1; p.bias = w->b_ff1; p.out = ws + L.ff;
        if ((rc = hyb_launch_gemm(gg, dt, dt, EPI_GEGLU, st))) return rc;
    }
    {
        GemmGroup gg = one(M, C, 4 * C);
        GemmProblem& p = gg.p[0];
        p.a = ws + L.ff; p.w = w->w_ff2; p.bias = w->b_ff2; p.out = x_out; p.res = g; p.res2 = x_in; p.rows_per_gate = 1;
        if ((rc = hyb_launch_gemm(gg, dt, HYB_F32, EPI_GATE_RES, st))) return rc;
    }
    return HYB_OK;
}

extern "C" int hyb_groupnorm(const float* x, const float* gamma, const float* beta, float* out,
                             int batch, int tokens, int channels, int groups, float eps,
                             void* workspace, size_t workspace_bytes, void* stream) {
    HYB_REQUIRE(batch >= 0 && tokens >= 0 && channels > 0 && groups > 0 && channels % groups == 0, HYB_ERR_SHAPE,
                "hyb_groupnorm: bad sizes (channels %d, groups %d)", channels, groups);
    HYB_REQUIRE(batch <= 65535, HYB_ERR_SHAPE, "hyb_groupnorm: batch exceeds 65535");
    if (batch == 0 || tokens == 0) return HYB_OK;
    HYB_CHECK_PTR(x); HYB_CHECK_PTR(gamma); HYB_CHECK_PTR(beta); HYB_CHECK_PTR(out); HYB_CHECK_PTR(workspace);
    HYB_CHECK_ALIGN(x); HYB_CHECK_ALIGN(out); HYB_CHECK_ALIGN(workspace);
    HYB_REQUIRE(workspace_bytes >= hyb_groupnorm_scratch_bytes(batch, groups), HYB_ERR_WORKSPACE,
                "hyb_groupnorm: workspace of %zu bytes is smaller than the %zu required", workspace_bytes, hyb_groupnorm_scratch_bytes(batch, groups));
    return hyb_launch_groupnorm(x, gamma, beta, out, batch, tokens, channels, groups, eps, workspace, (hipStream_t)stream);
}

extern "C" size_t hyb_groupnorm_workspace_bytes(int batch, int groups) {
    if (batch <= 0 || groups <= 0) return 0;
    return hyb_groupnorm_scratch_bytes(batch, groups);
}

extern "C" int hyb_layernorm_affine(const float* x, const float* gamma, const float* beta, void* out,
                                    int rows, int hidden, float eps, hyb_dtype out_dtype, void* stream) {
    HYB_CHECK_DTYPE(out_dtype);
    HYB_REQUIRE(rows >= 0, HYB_ERR_SHAPE, "hyb_layernorm_affine: negative size");
    HYB_REQUIRE(hidden > 0 && hidden % 4 == 0 && hidden <= 2048, HYB_ERR_SHAPE,
                "hyb_layernorm_affine: hidden %d must be a positive multiple of 4, at most 2048", hidden);
    if (rows == 0) return HYB_OK;
    HYB_CHECK_PTR(x); HYB_CHECK_PTR(gamma); HYB_CHECK_PTR(beta); HYB_CHECK_PTR(out);
    HYB_CHECK_ALIGN(x); HYB_CHECK_ALIGN(gamma); HYB_CHECK_ALIGN(beta); HYB_CHECK_ALIGN(out);
    return hyb_launch_layernorm(x, beta, gamma, 0, out, 1, rows, hidden, eps, out_dtype, true, (hipStream_t)stream);
}
