// Plain LDS-tiled FMA GEMM: out = epilogue(A W^T + bias) for any shape, fp32 or bf16 operands,
// fp32 accumulation in a fixed k order.  It is the fp32 (reference-precision) path of the
// denoiser forward and the fallback for shapes the MFMA kernel does not take.
#include "gemm.h"

namespace {

constexpr int TS = 64;   // tile rows = tile cols
constexpr int BK = 16;

template <typename T, typename OT, bool GEGLU>
__global__ __launch_bounds__(256) void gemm_simple_kernel(GemmGroup g, int epi, int tiles_m0) {
    __shared__ float As[BK][TS + 4];
    __shared__ float Ws[GEGLU ? 2 : 1][BK][TS + 4];
    const int pi = (int)blockIdx.y >= tiles_m0 ? 1 : 0;
    const GemmProblem& p = g.p[pi];
    const int row0 = ((int)blockIdx.y - (pi ? tiles_m0 : 0)) * TS;
    const int col0 = blockIdx.x * TS;
    const int n = g.n, k = g.k, m = p.m;
    const T* A = static_cast<const T*>(p.a);
    const T* W = static_cast<const T*>(p.w);
    const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
    const int lr = threadIdx.x / 4, lk = (threadIdx.x % 4) * 4;
    float acc[GEGLU ? 2 : 1][4][4] = {};
    for (int k0 = 0; k0 < k; k0 += BK) {
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const int kk = k0 + lk + j;
            const int ar = row0 + lr, wr = col0 + lr;
            As[lk + j][lr] = (ar < m && kk < k) ? to_f32<T>(A[(size_t)ar * k + kk]) : 0.f;
            Ws[0][lk + j][lr] = (wr < n && kk < k) ? to_f32<T>(W[(size_t)wr * k + kk]) : 0.f;
            if constexpr (GEGLU) Ws[1][lk + j][lr] = (wr < n && kk < k) ? to_f32<T>(W[(size_t)(n + wr) * k + kk]) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK; kk++) {
            float a[4], w[GEGLU ? 2 : 1][4];
#pragma unroll
            for (int i = 0; i < 4; i++) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int h = 0; h < (GEGLU ? 2 : 1); h++)
#pragma unroll
                for (int j = 0; j < 4; j++) w[h][j] = Ws[h][kk][tx * 4 + j];
#pragma unroll
            for (int h = 0; h < (GEGLU ? 2 : 1); h++)
#pragma unroll
                for (int i = 0; i < 4; i++)
#pragma unroll
                    for (int j = 0; j < 4; j++) acc[h][i][j] = fmaf(a[i], w[h][j], acc[h][i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const int r = row0 + ty * 4 + i;
        if (r >= m) continue;
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const int c = col0 + tx * 4 + j;
            if (c >= n) continue;
            float v = acc[0][i][j] + (p.bias ? p.bias[c] : 0.f);
            if constexpr (GEGLU) {
                const float gt = acc[1][i][j] + (p.bias ? p.bias[n + c] : 0.f);
                v *= gelu_erf_f(gt);
                static_cast<OT*>(p.out)[(size_t)r * n + c] = from_f32<OT>(v);
            } else {
                gemm_store_scalar<OT>(p, epi, n, r, c, v);
            }
        }
    }
}

template <typename T, typename OT>
int launch(const GemmGroup& g, int epi, hipStream_t st) {
    const int tiles_m0 = (g.p[0].m + TS - 1) / TS;
    const int tiles_m1 = g.count > 1 ? (g.p[1].m + TS - 1) / TS : 0;
    if (tiles_m0 + tiles_m1 == 0 || g.n == 0) return HYB_OK;
    dim3 grid((g.n + TS - 1) / TS, tiles_m0 + tiles_m1), block(256);
    HYB_REQUIRE(grid.y <= 65535, HYB_ERR_SHAPE, "gemm: too many row tiles (%u)", grid.y);
    char name[96];
    snprintf(name, sizeof(name), "gemm_simple.epi%d.n%d.k%d", epi, g.n, g.k);
    double rows = g.p[0].m + (g.count > 1 ? g.p[1].m : 0);
    HybTraceScope trace(name, "flop", 2.0 * rows * g.n * g.k * (epi == EPI_GEGLU ? 2 : 1), st);
    if (epi == EPI_GEGLU) hipLaunchKernelGGL((gemm_simple_kernel<T, OT, true>), grid, block, 0, st, g, epi, tiles_m0);
    else hipLaunchKernelGGL((gemm_simple_kernel<T, OT, false>), grid, block, 0, st, g, epi, tiles_m0);
    return hyb_check_launch("gemm_simple");
}

}  // namespace

int hyb_launch_gemm_simple(const GemmGroup& g, hyb_dtype in_dtype, hyb_dtype out_dtype, int epi, hipStream_t st) {
    if (in_dtype == HYB_F32) return out_dtype == HYB_F32 ? launch<float, float>(g, epi, st) : launch<float, bf16_t>(g, epi, st);
    return out_dtype == HYB_F32 ? launch<bf16_t, float>(g, epi, st) : launch<bf16_t, bf16_t>(g, epi, st);
}

int hyb_launch_gemm(const GemmGroup& g, hyb_dtype in_dtype, hyb_dtype out_dtype, int epi, hipStream_t st) {
    if (in_dtype == HYB_BF16) {
        const int rc = hyb_launch_gemm_mfma(g, out_dtype, epi, st);
        if (rc >= 0) return rc;
    }
    return hyb_launch_gemm_simple(g, in_dtype, out_dtype, epi, st);
}

extern "C" int hyb_linear(const void* a, const void* w, const float* bias, void* out, int m, int n, int k,
                          hyb_dtype dtype, hyb_dtype out_dtype, hyb_epilogue epi,
                          const float* residual, const float* gate, int rows_per_gate, size_t gate_stride,
                          void* stream) {
    HYB_CHECK_DTYPE(dtype); HYB_CHECK_DTYPE(out_dtype);
    HYB_REQUIRE((epi >= HYB_EPI_BIAS && epi <= HYB_EPI_GATE_RESIDUAL) || epi == HYB_EPI_GEGLU, HYB_ERR_DTYPE, "hyb_linear: unknown epilogue %d", (int)epi);
    HYB_REQUIRE(m >= 0 && n >= 0 && k >= 0, HYB_ERR_SHAPE, "hyb_linear: negative size");
    if (m == 0 || n == 0) return HYB_OK;
    HYB_CHECK_PTR(a); HYB_CHECK_PTR(w); HYB_CHECK_PTR(out);
    HYB_CHECK_ALIGN(a); HYB_CHECK_ALIGN(w); HYB_CHECK_ALIGN(out); HYB_CHECK_ALIGN(bias);
    GemmGroup g = {};
    g.count = 1; g.n = n; g.k = k;
    GemmProblem& p = g.p[0];
    p.a = a; p.w = w; p.bias = bias; p.out = out; p.m = m;
    if (epi == HYB_EPI_GATE_RESIDUAL) {
        HYB_REQUIRE(out_dtype == HYB_F32, HYB_ERR_DTYPE, "hyb_linear: HYB_EPI_GATE_RESIDUAL needs an fp32 output");
        HYB_CHECK_PTR(residual); HYB_CHECK_ALIGN(residual); HYB_CHECK_ALIGN(gate);
        HYB_REQUIRE(gate == nullptr || rows_per_gate > 0, HYB_ERR_SHAPE, "hyb_linear: rows_per_gate must be positive");
        p.res = residual; p.gate = gate; p.rows_per_gate = rows_per_gate > 0 ? rows_per_gate : 1; p.gate_stride = gate_stride;
    }
    return hyb_launch_gemm(g, dtype, out_dtype, (int)epi, (hipStream_t)stream);
}
