// Internal GEMM interface of libhyb: out = epilogue(A W^T + bias), A [m, k] and W [n, k] both
// k-contiguous.  Up to kMaxGroup independent problems with the same (n, k) and epilogue kind run
// in ONE launch (the image- and text-stream GEMMs of a joint block have different weights and
// row counts but the same shape otherwise).
#pragma once
#include "common.h"

enum GemmEpi {
    EPI_BIAS = 0,        // out[r, c] = acc + bias[c]
    EPI_GELU_TANH = 1,   // out[r, c] = GELUtanh(acc + bias[c])
    EPI_SILU = 2,        // out[r, c] = SiLU(acc + bias[c])
    EPI_GATE_RES = 3,    // out[r, c] (fp32) = res[r, c] (+ res2[r, c]) + gate[(r / rows_per_gate) * gate_stride + c] * (acc + bias[c])
    EPI_QKV = 4,         // scatter (acc + bias[c]) to head-major q / k / v (n = 1, 2 or 3 times heads * 64)
    EPI_GEGLU = 5        // out[r, c] = (acc_u + bias[c]) * GELUerf(acc_g + bias[n + c]), W rows [u; g] (2n rows)
};

constexpr int kMaxGroup = 2;

struct GemmProblem {
    const void* a;       // [m, k]
    const void* w;       // [n, k]  (EPI_GEGLU: [2n, k])
    const float* bias;   // [n] or nullptr
    void* out;           // [m, n] of out dtype (unused for EPI_QKV)
    int m;
    // EPI_GATE_RES
    const float* res;
    const float* res2;   // optional second residual
    const float* gate;   // nullptr -> 1
    int rows_per_gate;
    size_t gate_stride;
    // EPI_QKV: row r = (b, t) with t < tokens; column c = (which, head, i), n = 3 * heads * 64;
    // element -> {q,k,v}[((b * heads + head) * n_total) + tok_offset + t][i]
    void* q; void* k; void* v;
    int tokens, tok_offset, n_total, heads;
    float q_scale;       // EPI_QKV: the q part is multiplied by this before it is rounded (0 means 1): lets the attention
                         // kernel take queries that already carry softmax scale x log2(e)
};

struct GemmGroup {
    GemmProblem p[kMaxGroup];
    int count;
    int n, k;
    // Scratch for the MFMA path's k split (single problem, few tiles, long k: see gemm_mfma.hip), or nullptr.
    void* splitk_ws;
    size_t splitk_bytes;
};

// Plain tiled FMA kernel: any shape, fp32 or bf16 operands, fp32 accumulation.
int hyb_launch_gemm_simple(const GemmGroup& g, hyb_dtype in_dtype, hyb_dtype out_dtype, int epi, hipStream_t st);
// bf16 MFMA kernel (k % 64 == 0, n % 8 == 0); returns -1 if the shape is not supported.
int hyb_launch_gemm_mfma(const GemmGroup& g, hyb_dtype out_dtype, int epi, hipStream_t st);
// Large-tile bf16 MFMA kernel (256 x 128 tiles, one workgroup per CU).  Same accumulation order as the kernel above, hence
// the same bits per token.  -1 when the shape or the epilogue has no large-tile form.
int hyb_launch_gemm_mfma_big(const GemmGroup& g, hyb_dtype out_dtype, int epi, hipStream_t st);
// Dispatch: MFMA for bf16 when supported, else the plain kernel.
int hyb_launch_gemm(const GemmGroup& g, hyb_dtype in_dtype, hyb_dtype out_dtype, int epi, hipStream_t st);

// Scalar epilogue shared by both kernels' tails (v = acc + bias already applied by the caller
// where the epilogue needs it).
template <typename OT>
__device__ __forceinline__ void gemm_store_scalar(const GemmProblem& p, int epi, int n, int r, int c, float v) {
    if (epi == EPI_QKV) {
        const int hd = p.heads * 64;
        const int which = c / hd, cc = c % hd, head = cc / 64, i = cc % 64;
        const int b = r / p.tokens, t = r % p.tokens;
        if (which == 0 && p.q_scale != 0.f) v *= p.q_scale;
        OT* base = static_cast<OT*>(which == 0 ? p.q : (which == 1 ? p.k : p.v));
        base[(((size_t)b * p.heads + head) * p.n_total + p.tok_offset + t) * 64 + i] = from_f32<OT>(v);
        return;
    }
    const size_t o = (size_t)r * n + c;
    if (epi == EPI_GELU_TANH) v = gelu_tanh_f(v);
    else if (epi == EPI_SILU) v = silu_f(v);
    else if (epi == EPI_GATE_RES) {
        const float g = p.gate ? p.gate[(size_t)(r / p.rows_per_gate) * p.gate_stride + c] : 1.f;
        v = fmaf(g, v, p.res[o]);
        if (p.res2) v += p.res2[o];
    }
    static_cast<OT*>(p.out)[o] = from_f32<OT>(v);
}
