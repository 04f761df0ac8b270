// Plain softmax attention, fp32 math: the reference-precision path (fp32 workloads).
// One wave per query row.  Keys are taken 64 at a time: lane l scores key j0 + l against the
// query (held in LDS), the running maximum / normaliser follow the usual streaming-softmax
// recurrence, and lane i accumulates output feature i.
#include "attention.h"

namespace {

template <typename T>
__global__ __launch_bounds__(256) void attention_simple_kernel(AttnArgs a) {
    __shared__ float qs[4][64];
    const int wave = threadIdx.x / HYB_WAVE, lane = threadIdx.x % HYB_WAVE;
    const int row = blockIdx.x * 4 + wave;
    const int h = blockIdx.y, b = blockIdx.z;
    const bool active = row < a.n_q;
    const size_t bh = (size_t)b * a.heads + h;
    const T* q = static_cast<const T*>(a.q) + (bh * (a.q_stride ? a.q_stride : a.n_q) + (active ? row : 0)) * 64;
    const T* k = static_cast<const T*>(a.k) + bh * a.n_kv * 64;
    const T* v = static_cast<const T*>(a.v) + bh * a.n_kv * 64;
    qs[wave][lane] = to_f32<T>(q[lane]);
    __syncthreads();
    if (!active) return;
    float m = -__builtin_inff(), l = 0.f, acc = 0.f;
    for (int j0 = 0; j0 < a.n_kv; j0 += 64) {
        const int j = j0 + lane;
        float s = -__builtin_inff();
        if (j < a.n_kv) {
            const T* kr = k + (size_t)j * 64;
            float d = 0.f;
#pragma unroll 8
            for (int i = 0; i < 64; i++) d = fmaf(qs[wave][i], to_f32<T>(kr[i]), d);
            s = d * a.scale;
        }
        const float m_new = fmaxf(m, wave_max(s));
        const float corr = expf(m - m_new);          // first tile: exp(-inf) = 0
        const float p = expf(s - m_new);             // masked keys: exp(-inf) = 0
        l = l * corr + wave_sum(p);
        acc *= corr;
        const int cnt = min(64, a.n_kv - j0);
        for (int jj = 0; jj < cnt; jj++) {
            const float pj = __shfl(p, jj, 64);
            acc = fmaf(pj, to_f32<T>(v[(size_t)(j0 + jj) * 64 + lane]), acc);
        }
        m = m_new;
    }
    const int hd = a.heads * 64;
    T* o;
    if (row < a.split) o = static_cast<T*>(a.o) + ((size_t)b * a.split + row) * hd;
    else o = static_cast<T*>(a.o2) + ((size_t)b * (a.n_q - a.split) + (row - a.split)) * hd;
    o[h * 64 + lane] = from_f32<T>(acc / l);
}

}  // namespace

int hyb_launch_attention_simple(const AttnArgs& a, hyb_dtype dtype, hipStream_t st) {
    dim3 grid((a.n_q + 3) / 4, a.heads, a.batch), block(256);
    HybTraceScope trace("attention_simple", "flop", 4.0 * a.batch * a.heads * (double)a.n_q * a.n_kv * 64, st);
    if (dtype == HYB_F32) hipLaunchKernelGGL((attention_simple_kernel<float>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((attention_simple_kernel<bf16_t>), grid, block, 0, st, a);
    return hyb_check_launch("attention_simple");
}

int hyb_launch_attention(const AttnArgs& a, hyb_dtype dtype, hipStream_t st) {
    if (a.batch == 0 || a.n_q == 0 || a.heads == 0) return HYB_OK;
    if (dtype == HYB_BF16) return hyb_launch_attention_mfma(a, st);
    return hyb_launch_attention_simple(a, dtype, st);
}

namespace {
int joint_attention(const char* who, const void* q, const void* k, const void* v, void* o,
                    int batch, int heads, int n_q, int n_kv, int head_dim, float scale,
                    hyb_dtype dtype, void* workspace, size_t workspace_bytes, bool with_ws, bool prescaled, void* stream) {
    HYB_CHECK_DTYPE(dtype);
    HYB_REQUIRE(batch >= 0 && heads >= 0 && n_q >= 0 && n_kv >= 0, HYB_ERR_SHAPE, "%s: negative size", who);
    HYB_REQUIRE(head_dim == 64, HYB_ERR_SHAPE, "%s: head_dim %d is not supported (only 64)", who, head_dim);
    HYB_REQUIRE(batch <= 65535 && heads <= 65535, HYB_ERR_SHAPE, "%s: batch and heads must be at most 65535", who);
    if (batch == 0 || heads == 0 || n_q == 0) return HYB_OK;
    HYB_REQUIRE(n_kv > 0, HYB_ERR_SHAPE, "%s: n_kv == 0 with n_q > 0 (softmax over an empty set)", who);
    HYB_CHECK_PTR(q); HYB_CHECK_PTR(k); HYB_CHECK_PTR(v); HYB_CHECK_PTR(o);
    HYB_CHECK_ALIGN(q); HYB_CHECK_ALIGN(k); HYB_CHECK_ALIGN(v); HYB_CHECK_ALIGN(o);
    AttnArgs a = {q, k, v, o, nullptr, n_q, batch, heads, n_q, n_kv, scale > 0.f ? scale : 0.125f};
    if (prescaled) {
        // q carries scale x log2(e): the bf16 kernel exponentiates the raw scores in base 2; the fp32 kernel, which
        // exponentiates scale x score in base e, gets scale = ln 2
        a.prescaled = dtype == HYB_BF16;
        a.scale = 0.6931471805599453f;
    }
    if (with_ws) {
        const size_t need = hyb_joint_attention_workspace_bytes(batch, heads, n_q, dtype);
        if (need > 0) {
            HYB_CHECK_PTR(workspace); HYB_CHECK_ALIGN(workspace);
            HYB_REQUIRE(workspace_bytes >= need, HYB_ERR_WORKSPACE, "%s: workspace of %zu bytes is smaller than the %zu required", who, workspace_bytes, need);
            a.part = static_cast<float*>(workspace);
        }
    }
    return hyb_launch_attention(a, dtype, (hipStream_t)stream);
}
}  // namespace

extern "C" int hyb_joint_attention(const void* q, const void* k, const void* v, void* o,
                                   int batch, int heads, int n_q, int n_kv, int head_dim, float scale,
                                   hyb_dtype dtype, void* stream) {
    return joint_attention("hyb_joint_attention", q, k, v, o, batch, heads, n_q, n_kv, head_dim, scale, dtype, nullptr, 0, false, false, stream);
}

extern "C" size_t hyb_joint_attention_workspace_bytes(int batch, int heads, int n_q, hyb_dtype dtype) {
    if (dtype != HYB_BF16 || batch <= 0 || heads <= 0 || n_q <= 0) return 0;
    return hyb_align_up(hyb_attention_split_bytes(batch, heads, n_q), 256);
}

extern "C" int hyb_joint_attention_ws(const void* q, const void* k, const void* v, void* o,
                                      int batch, int heads, int n_q, int n_kv, int head_dim, float scale,
                                      hyb_dtype dtype, void* workspace, size_t workspace_bytes, void* stream) {
    return joint_attention("hyb_joint_attention_ws", q, k, v, o, batch, heads, n_q, n_kv, head_dim, scale, dtype, workspace, workspace_bytes, true, false, stream);
}

extern "C" int hyb_joint_attention_prescaled(const void* q, const void* k, const void* v, void* o,
                                             int batch, int heads, int n_q, int n_kv, int head_dim,
                                             hyb_dtype dtype, void* workspace, size_t workspace_bytes, void* stream) {
    return joint_attention("hyb_joint_attention_prescaled", q, k, v, o, batch, heads, n_q, n_kv, head_dim, 0.f, dtype, workspace, workspace_bytes, true, true, stream);
}
