// bf16 MFMA GEMM for gfx950: out = epilogue(A W^T + bias), A [m, k] tokens x features-in,
// W [n, k] features-out x features-in, fp32 accumulation in v_mfma_f32_32x32x16_bf16.
//
// Tiling: a workgroup of 4 waves (2 x 2) owns a BM x BN output tile (BM = 64 TM tokens,
// BN = 64 TN features); each wave owns TM x TN MFMA tiles of 32 x 32.  The weight fragment is
// the MFMA "A" operand and the token fragment the "B" operand, so that the 16 accumulator
// registers of a lane run along the OUTPUT FEATURE axis (4 consecutive features per group of
// 4 registers, one token per lane): bias / gate / residual / output are then moved as 8- or
// 16-byte vectors.  Both operands are k-contiguous, so global -> LDS copies are 16-byte
// vectors (8 lanes cover one 128-byte row of a 64-wide k slab), and LDS rows are padded by
// 16 bytes so that the 16-byte fragment reads of 16 consecutive rows hit distinct banks.
// The next k slab is fetched into registers while the current one is multiplied.
//
// Up to two problems with the same (n, k) share a launch (image and text stream of a joint
// block).  Ragged edges: row / feature indices are clamped on load and masked on store.
// The reduction order over k is fixed, and a token's result does not depend on which tile
// row it falls in, so results are deterministic and batch-invariant.
#include "gemm.h"

namespace {

constexpr int BK = 64;
constexpr int LDS_STRIDE = BK + 8;   // bf16 elements per LDS row (144 bytes)

template <int TM, int TN>
struct Tile {
    static constexpr int BM = 64 * TM;
    static constexpr int BN = 64 * TN;
    static constexpr int A_VECS = BM / 32;   // 16-byte vectors per thread per slab
    static constexpr int W_VECS = BN / 32;
};

template <typename OT> __device__ __forceinline__ void store4(OT* p, const f32x4& v);
template <> __device__ __forceinline__ void store4<float>(float* p, const f32x4& v) { *reinterpret_cast<f32x4*>(p) = v; }
template <> __device__ __forceinline__ void store4<bf16_t>(bf16_t* p, const f32x4& v) {
    bf16x4 o = {(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
    *reinterpret_cast<bf16x4*>(p) = o;
}

template <int TM, int TN, typename OT, int EPI>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(GemmGroup g, int tiles_n, int tiles0) {
    using T = Tile<TM, TN>;
    __shared__ __attribute__((aligned(16))) bf16_t As[T::BM * LDS_STRIDE];
    __shared__ __attribute__((aligned(16))) bf16_t Ws[T::BN * LDS_STRIDE];

    int tile = blockIdx.x;
    const int pi = tile >= tiles0 ? 1 : 0;
    if (pi) tile -= tiles0;
    const GemmProblem& p = g.p[pi];
    const int row0 = (tile / tiles_n) * T::BM;
    const int col0 = (tile % tiles_n) * T::BN;
    const int m = p.m, n = g.n, k = g.k;
    const bf16_t* A = static_cast<const bf16_t*>(p.a);
    const bf16_t* W = static_cast<const bf16_t*>(p.w);

    const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
    const int wt = wave % 2, wf = wave / 2;          // wave position: tokens, features
    const int ld_row = tid / 8, ld_vec = tid % 8;    // global -> LDS copy role

    const bf16_t* a_src[T::A_VECS];
    const bf16_t* w_src[T::W_VECS];
#pragma unroll
    for (int i = 0; i < T::A_VECS; i++) a_src[i] = A + (size_t)min(row0 + ld_row + 32 * i, m - 1) * k + ld_vec * 8;
#pragma unroll
    for (int i = 0; i < T::W_VECS; i++) w_src[i] = W + (size_t)min(col0 + ld_row + 32 * i, n - 1) * k + ld_vec * 8;

    f32x16 acc[TN][TM];
#pragma unroll
    for (int fn = 0; fn < TN; fn++)
#pragma unroll
        for (int tm = 0; tm < TM; tm++)
#pragma unroll
            for (int i = 0; i < 16; i++) acc[fn][tm][i] = 0.f;

    bf16x8 a_reg[T::A_VECS], w_reg[T::W_VECS];
#pragma unroll
    for (int i = 0; i < T::A_VECS; i++) a_reg[i] = *reinterpret_cast<const bf16x8*>(a_src[i]);
#pragma unroll
    for (int i = 0; i < T::W_VECS; i++) w_reg[i] = *reinterpret_cast<const bf16x8*>(w_src[i]);

    const int frag_off = (lane % 32) * LDS_STRIDE + (lane / 32) * 8;
    const int nslab = k / BK;
    for (int s = 0; s < nslab; s++) {
#pragma unroll
        for (int i = 0; i < T::A_VECS; i++) *reinterpret_cast<bf16x8*>(&As[(ld_row + 32 * i) * LDS_STRIDE + ld_vec * 8]) = a_reg[i];
#pragma unroll
        for (int i = 0; i < T::W_VECS; i++) *reinterpret_cast<bf16x8*>(&Ws[(ld_row + 32 * i) * LDS_STRIDE + ld_vec * 8]) = w_reg[i];
        __syncthreads();
        if (s + 1 < nslab) {
#pragma unroll
            for (int i = 0; i < T::A_VECS; i++) a_reg[i] = *reinterpret_cast<const bf16x8*>(a_src[i] + (size_t)(s + 1) * BK);
#pragma unroll
            for (int i = 0; i < T::W_VECS; i++) w_reg[i] = *reinterpret_cast<const bf16x8*>(w_src[i] + (size_t)(s + 1) * BK);
        }
#pragma unroll
        for (int kk = 0; kk < BK / 16; kk++) {
            bf16x8 af[TM], wfr[TN];
#pragma unroll
            for (int tm = 0; tm < TM; tm++)
                af[tm] = *reinterpret_cast<const bf16x8*>(&As[(wt * 32 * TM + tm * 32) * LDS_STRIDE + frag_off + kk * 16]);
#pragma unroll
            for (int fn = 0; fn < TN; fn++)
                wfr[fn] = *reinterpret_cast<const bf16x8*>(&Ws[(wf * 32 * TN + fn * 32) * LDS_STRIDE + frag_off + kk * 16]);
#pragma unroll
            for (int fn = 0; fn < TN; fn++)
#pragma unroll
                for (int tm = 0; tm < TM; tm++)
                    acc[fn][tm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wfr[fn], af[tm], acc[fn][tm], 0, 0, 0);
        }
        __syncthreads();
    }

    // Epilogue.  Register i of tile (fn, tm): feature = f_base + 8 (i / 4) + 4 (lane / 32) + i % 4,
    // token = r_base + lane % 32.
#pragma unroll
    for (int tm = 0; tm < TM; tm++) {
        const int r = row0 + wt * 32 * TM + tm * 32 + lane % 32;
        if (r >= m) continue;
        size_t qkv_row = 0;
        int qb = 0;
        if constexpr (EPI == EPI_QKV) {
            qb = r / p.tokens;
            qkv_row = (size_t)p.tok_offset + (r - qb * p.tokens);
        }
        const float* gate_row = nullptr;
        if constexpr (EPI == EPI_GATE_RES) {
            if (p.gate) gate_row = p.gate + (size_t)(r / p.rows_per_gate) * p.gate_stride;
        }
#pragma unroll
        for (int fn = 0; fn < TN; fn++) {
#pragma unroll
            for (int gi = 0; gi < 4; gi++) {
                const int f = col0 + wf * 32 * TN + fn * 32 + 8 * gi + 4 * (lane / 32);
                if (f >= n) continue;
                f32x4 v = {acc[fn][tm][4 * gi], acc[fn][tm][4 * gi + 1], acc[fn][tm][4 * gi + 2], acc[fn][tm][4 * gi + 3]};
                if (p.bias) v += *reinterpret_cast<const f32x4*>(p.bias + f);
                if constexpr (EPI == EPI_QKV) {
                    const int hd = p.heads * 64;
                    const int which = f / hd, cc = f - which * hd, head = cc / 64, i0 = cc % 64;
                    OT* base = static_cast<OT*>(which == 0 ? p.q : (which == 1 ? p.k : p.v));
                    store4<OT>(base + (((size_t)qb * p.heads + head) * p.n_total + qkv_row) * 64 + i0, v);
                } else {
                    const size_t o = (size_t)r * n + f;
                    if constexpr (EPI == EPI_GELU_TANH) {
#pragma unroll
                        for (int j = 0; j < 4; j++) v[j] = gelu_tanh_f(v[j]);
                    } else if constexpr (EPI == EPI_SILU) {
#pragma unroll
                        for (int j = 0; j < 4; j++) v[j] = silu_f(v[j]);
                    } else if constexpr (EPI == EPI_GATE_RES) {
                        const f32x4 res = *reinterpret_cast<const f32x4*>(p.res + o);
                        if (gate_row) {
                            const f32x4 gt = *reinterpret_cast<const f32x4*>(gate_row + f);
#pragma unroll
                            for (int j = 0; j < 4; j++) v[j] = fmaf(gt[j], v[j], res[j]);
                        } else {
                            v += res;
                        }
                    }
                    store4<OT>(static_cast<OT*>(p.out) + o, v);
                }
            }
        }
    }
}

template <int TM, int TN, typename OT, int EPI>
int launch_tile(const GemmGroup& g, hipStream_t st) {
    using T = Tile<TM, TN>;
    const int tiles_n = (g.n + T::BN - 1) / T::BN;
    const int tiles0 = ((g.p[0].m + T::BM - 1) / T::BM) * tiles_n;
    const int tiles1 = g.count > 1 ? ((g.p[1].m + T::BM - 1) / T::BM) * tiles_n : 0;
    if (tiles0 + tiles1 == 0) return HYB_OK;
    char name[96];
    snprintf(name, sizeof(name), "gemm_mfma_%dx%d.epi%d.n%d.k%d", T::BM, T::BN, EPI, g.n, g.k);
    double rows = g.p[0].m + (g.count > 1 ? g.p[1].m : 0);
    HybTraceScope trace(name, "flop", 2.0 * rows * g.n * g.k, st);
    GemmGroup gg = g;
    if (tiles0 == 0) {  // keep problem 0 non-empty so that the tile -> problem split stays simple
        gg.p[0] = g.p[1];
        gg.count = 1;
        hipLaunchKernelGGL((gemm_mfma_kernel<TM, TN, OT, EPI>), dim3(tiles1), dim3(256), 0, st, gg, tiles_n, tiles1);
    } else {
        hipLaunchKernelGGL((gemm_mfma_kernel<TM, TN, OT, EPI>), dim3(tiles0 + tiles1), dim3(256), 0, st, gg, tiles_n, tiles0);
    }
    return hyb_check_launch("gemm_mfma");
}

template <typename OT, int EPI>
int launch_epi(const GemmGroup& g, hipStream_t st) {
    return launch_tile<2, 2, OT, EPI>(g, st);
}

}  // namespace

int hyb_launch_gemm_mfma(const GemmGroup& g, hyb_dtype out_dtype, int epi, hipStream_t st) {
    if (g.k <= 0 || g.k % BK != 0 || g.n % 8 != 0 || epi == EPI_GEGLU) return -1;
    for (int i = 0; i < g.count; i++) {
        const GemmProblem& p = g.p[i];
        if (epi == EPI_GATE_RES && p.gate && (p.gate_stride % 4 != 0)) return -1;
        if (epi == EPI_QKV && g.n != 3 * p.heads * 64) return -1;
    }
    const bool f32 = out_dtype == HYB_F32;
    switch (epi) {
        case EPI_BIAS: return f32 ? launch_epi<float, EPI_BIAS>(g, st) : launch_epi<bf16_t, EPI_BIAS>(g, st);
        case EPI_GELU_TANH: return f32 ? launch_epi<float, EPI_GELU_TANH>(g, st) : launch_epi<bf16_t, EPI_GELU_TANH>(g, st);
        case EPI_SILU: return f32 ? launch_epi<float, EPI_SILU>(g, st) : launch_epi<bf16_t, EPI_SILU>(g, st);
        case EPI_GATE_RES: return f32 ? launch_epi<float, EPI_GATE_RES>(g, st) : -1;
        case EPI_QKV: return f32 ? -1 : launch_epi<bf16_t, EPI_QKV>(g, st);
        default: return -1;
    }
}
