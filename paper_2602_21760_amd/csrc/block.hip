// Host-side composition of one joint image+text transformer block from the library's kernels
// (the unit of work inside the denoiser f_theta of one guidance branch, Sec. 4.1).
// Seven launches per block: LN+modulate (both streams, one launch) -> grouped QKV GEMM with head-major
// scatter -> joint attention -> grouped out-projection with gate * y + residual -> LN+modulate ->
// grouped fc1 with GELU -> grouped fc2 with gate * y + residual.
#include "attention.h"
#include "gemm.h"

int hyb_launch_layernorm(const float* x, const float* shift, const float* scale, size_t mod_stride, void* out,
                         int batch, int tokens, int hidden, float eps, hyb_dtype out_dtype, bool affine, hipStream_t st);
int hyb_launch_layernorm_pair(const float* const x[2], const float* const shift[2], const float* const scale[2],
                              size_t mod_stride, void* const out[2], int batch, const int tokens[2], int hidden,
                              float eps, hyb_dtype out_dtype, hipStream_t st);

namespace {

struct BlockLayout {
    size_t h_img, h_txt, q, k, v, o_img, o_txt, mlp_img, mlp_txt, attn_part, total;
};

BlockLayout block_layout(const hyb_block_desc& d) {
    const size_t es = hyb_dtype_size(d.dtype);
    const size_t B = d.batch, Ni = d.n_img, Nt = d.n_txt, D = d.hidden, N = Ni + Nt;
    BlockLayout L;
    size_t off = 0;
    auto take = [&](size_t elems) {
        const size_t o = off;
        off += hyb_align_up(elems * es, 256);
        return o;
    };
    L.h_img = take(B * Ni * D);
    L.h_txt = take(B * Nt * D);
    L.q = take(B * N * D);
    L.k = take(B * N * D);
    L.v = take(B * N * D);
    L.o_img = take(B * Ni * D);
    L.o_txt = take(B * Nt * D);
    L.mlp_img = take(B * Ni * D * d.mlp_ratio);
    L.mlp_txt = take(B * Nt * D * d.mlp_ratio);
    // scratch of the attention kernel's split tail (bf16 path only; sized for image-only queries too, which
    // never need more)
    L.attn_part = off;
    if (d.dtype == HYB_BF16) {
        const size_t joint = hyb_attention_split_bytes(d.batch, d.heads, d.n_img + d.n_txt);
        const size_t img_only = hyb_attention_split_bytes(d.batch, d.heads, d.n_img);
        off += hyb_align_up(joint > img_only ? joint : img_only, 256);
    }
    L.total = off;
    return L;
}

int check_desc(const char* who, const hyb_block_desc* d) {
    HYB_CHECK_PTR(d);
    HYB_CHECK_DTYPE(d->dtype);
    HYB_REQUIRE(d->batch >= 0 && d->n_img >= 0 && d->n_txt >= 0, HYB_ERR_SHAPE, "%s: negative size", who);
    HYB_REQUIRE(d->head_dim == 64, HYB_ERR_SHAPE, "%s: head_dim %d is not supported (only 64)", who, d->head_dim);
    HYB_REQUIRE(d->heads > 0 && d->hidden == d->heads * d->head_dim, HYB_ERR_SHAPE, "%s: hidden %d != heads %d * head_dim %d", who, d->hidden, d->heads, d->head_dim);
    HYB_REQUIRE(d->hidden <= 2048, HYB_ERR_SHAPE, "%s: hidden %d exceeds 2048", who, d->hidden);
    HYB_REQUIRE(d->mlp_ratio > 0, HYB_ERR_SHAPE, "%s: mlp_ratio must be positive", who);
    HYB_REQUIRE(d->batch <= 65535, HYB_ERR_SHAPE, "%s: batch exceeds 65535", who);
    return HYB_OK;
}

}  // namespace

extern "C" size_t hyb_block_workspace_bytes(const hyb_block_desc* desc) {
    if (check_desc("hyb_block_workspace_bytes", desc) != HYB_OK) return 0;
    return block_layout(*desc).total;
}

extern "C" int hyb_block_forward(const hyb_block_desc* desc, const hyb_block_weights* weights,
                                 const float* x_img_in, const float* x_txt_in,
                                 const float* mod_img, const float* mod_txt, size_t mod_stride,
                                 float* x_img_out, float* x_txt_out,
                                 void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_desc("hyb_block_forward", desc);
    if (rc) return rc;
    HYB_CHECK_PTR(weights);
    const hyb_block_desc& d = *desc;
    const int B = d.batch, Ni = d.n_img, Nt = d.n_txt, D = d.hidden, N = Ni + Nt;
    if (B == 0 || N == 0) return HYB_OK;
    const bool has_img = Ni > 0, has_txt = Nt > 0;
    if (has_img) {
        HYB_CHECK_PTR(x_img_in); HYB_CHECK_PTR(x_img_out); HYB_CHECK_PTR(mod_img);
        HYB_CHECK_ALIGN(x_img_in); HYB_CHECK_ALIGN(x_img_out); HYB_CHECK_ALIGN(mod_img);
    }
    const bool txt_pre_only = d.txt_pre_only != 0 && has_txt;   // text: keys and values only, nothing written back
    if (has_txt) {
        HYB_CHECK_PTR(x_txt_in); HYB_CHECK_PTR(mod_txt);
        HYB_CHECK_ALIGN(x_txt_in); HYB_CHECK_ALIGN(mod_txt);
        if (!txt_pre_only) { HYB_CHECK_PTR(x_txt_out); HYB_CHECK_ALIGN(x_txt_out); }
    }
    HYB_REQUIRE(mod_stride % 4 == 0 && mod_stride >= (size_t)6 * D, HYB_ERR_SHAPE, "hyb_block_forward: mod_stride must be a multiple of 4 and at least 6 * hidden");
    const hyb_stream_weights* sw[2] = {&weights->img, &weights->txt};
    for (int s = 0; s < 2; s++) {
        if ((s == 0 && !has_img) || (s == 1 && !has_txt)) continue;
        const void* ptrs[8] = {sw[s]->w_qkv, sw[s]->w_out, sw[s]->w_fc1, sw[s]->w_fc2, sw[s]->b_qkv, sw[s]->b_out, sw[s]->b_fc1, sw[s]->b_fc2};
        for (int i = 0; i < 8; i++) {
            if (s == 1 && txt_pre_only && i != 0 && i != 4) continue;   // only the QKV projection is used
            HYB_REQUIRE(ptrs[i] != nullptr, HYB_ERR_NULL, "hyb_block_forward: a weight pointer of the %s stream is NULL", s ? "text" : "image");
            HYB_REQUIRE(((uintptr_t)ptrs[i] & 15u) == 0, HYB_ERR_ALIGN, "hyb_block_forward: a weight pointer of the %s stream is not 16-byte aligned", s ? "text" : "image");
        }
    }
    const BlockLayout L = block_layout(d);
    HYB_CHECK_PTR(workspace); HYB_CHECK_ALIGN(workspace);
    HYB_REQUIRE(workspace_bytes >= L.total, HYB_ERR_WORKSPACE, "hyb_block_forward: workspace of %zu bytes is smaller than the %zu required", workspace_bytes, L.total);

    hipStream_t st = (hipStream_t)stream;
    char* ws = static_cast<char*>(workspace);
    const hyb_dtype dt = d.dtype;
    void* h[2] = {ws + L.h_img, ws + L.h_txt};
    void* o[2] = {ws + L.o_img, ws + L.o_txt};
    void* mlp[2] = {ws + L.mlp_img, ws + L.mlp_txt};
    const float* xin[2] = {x_img_in, x_txt_in};
    float* xout[2] = {x_img_out, x_txt_out};
    const float* mod[2] = {mod_img, mod_txt};
    const int ntok[2] = {Ni, Nt};
    const int toff[2] = {0, Ni};

    // Problems of empty streams have m = 0 and cost nothing.  After the attention a "pre-only" text stream
    // is such an empty stream.
    const int ntok_post[2] = {Ni, txt_pre_only ? 0 : Nt};
    auto group = [&](int n, int k, const int* rows) {
        GemmGroup g = {};
        g.count = 2; g.n = n; g.k = k;
        for (int s = 0; s < 2; s++) g.p[s].m = B * rows[s];
        return g;
    };

    // 1. h = LN(x)(1 + scale1) + shift1
    {
        const float* sh[2] = {mod[0], mod[1]};
        const float* sc[2] = {mod[0] ? mod[0] + D : nullptr, mod[1] ? mod[1] + D : nullptr};
        if ((rc = hyb_launch_layernorm_pair(xin, sh, sc, mod_stride, h, B, ntok, D, d.ln_eps, dt, st))) return rc;
    }
    // 2. q, k, v = h Wqkv^T + b, scattered head-major into the joint (image first) sequence
    {
        GemmGroup g = group(3 * D, D, ntok);
        for (int s = 0; s < 2; s++) {
            GemmProblem& p = g.p[s];
            p.a = h[s]; p.w = sw[s]->w_qkv; p.bias = sw[s]->b_qkv;
            p.q = ws + L.q; p.k = ws + L.k; p.v = ws + L.v;
            p.tokens = ntok[s] > 0 ? ntok[s] : 1; p.tok_offset = toff[s]; p.n_total = N; p.heads = d.heads;
            // the bf16 attention kernel takes queries that already carry 1/sqrt(64) x log2(e) (one rounding either way)
            if (dt == HYB_BF16) p.q_scale = 0.125f * 1.4426950408889634f;
        }
        if ((rc = hyb_launch_gemm(g, dt, dt, EPI_QKV, st))) return rc;
    }
    // 3. joint attention; image rows go to o_img, text rows to o_txt
    {
        AttnArgs a = {ws + L.q, ws + L.k, ws + L.v, o[0], o[1], Ni, B, d.heads, N, N, 0.125f, N};
        if (L.total > L.attn_part) a.part = reinterpret_cast<float*>(ws + L.attn_part);
        if (!has_img) { a.o = o[1]; a.o2 = nullptr; a.split = N; }
        if (!has_txt) { a.o2 = nullptr; a.split = N; }
        if (txt_pre_only) { a.n_q = Ni; a.o2 = nullptr; a.split = Ni; }   // image queries only, joint keys
        a.prescaled = dt == HYB_BF16;
        if ((rc = hyb_launch_attention(a, dt, st))) return rc;
    }
    // 4. x = x + gate1 * (o Wout^T + b)
    {
        GemmGroup g = group(D, D, ntok_post);
        for (int s = 0; s < 2; s++) {
            GemmProblem& p = g.p[s];
            p.a = o[s]; p.w = sw[s]->w_out; p.bias = sw[s]->b_out; p.out = xout[s];
            p.res = xin[s]; p.gate = mod[s] ? mod[s] + 2 * D : nullptr; p.rows_per_gate = ntok[s] > 0 ? ntok[s] : 1; p.gate_stride = mod_stride;
        }
        if ((rc = hyb_launch_gemm(g, dt, HYB_F32, EPI_GATE_RES, st))) return rc;
    }
    // 5. h2 = LN(x)(1 + scale2) + shift2
    {
        const float* sh[2] = {mod[0] ? mod[0] + 3 * D : nullptr, mod[1] ? mod[1] + 3 * D : nullptr};
        const float* sc[2] = {mod[0] ? mod[0] + 4 * D : nullptr, mod[1] ? mod[1] + 4 * D : nullptr};
        if ((rc = hyb_launch_layernorm_pair(xout, sh, sc, mod_stride, h, B, ntok_post, D, d.ln_eps, dt, st))) return rc;
    }
    // 6. u = GELUtanh(h2 W1^T + b1)
    {
        GemmGroup g = group(d.mlp_ratio * D, D, ntok_post);
        for (int s = 0; s < 2; s++) {
            GemmProblem& p = g.p[s];
            p.a = h[s]; p.w = sw[s]->w_fc1; p.bias = sw[s]->b_fc1; p.out = mlp[s];
        }
        if ((rc = hyb_launch_gemm(g, dt, dt, EPI_GELU_TANH, st))) return rc;
    }
    // 7. x = x + gate2 * (u W2^T + b2)
    {
        GemmGroup g = group(D, d.mlp_ratio * D, ntok_post);
        for (int s = 0; s < 2; s++) {
            GemmProblem& p = g.p[s];
            p.a = mlp[s]; p.w = sw[s]->w_fc2; p.bias = sw[s]->b_fc2; p.out = xout[s];
            p.res = xout[s]; p.gate = mod[s] ? mod[s] + 5 * D : nullptr; p.rows_per_gate = ntok[s] > 0 ? ntok[s] : 1; p.gate_stride = mod_stride;
        }
        if ((rc = hyb_launch_gemm(g, dt, HYB_F32, EPI_GATE_RES, st))) return rc;
    }
    return HYB_OK;
}
