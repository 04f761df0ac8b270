// Flash-style joint attention for gfx950, bf16 operands, head_dim 64:
// o = softmax(q k^T * scale) v with a streaming (online) softmax, never materialising scores.
//
// A workgroup of 4 waves owns 128 query rows of one (batch, head); each wave owns 32 of them.
// Keys / values are streamed 64 at a time through double-buffered LDS tiles shared by the waves.
// Both contractions run on v_mfma_f32_32x32x16_bf16 in TRANSPOSED form:
//   S^T = K Q^T   (A operand: a K row per lane from LDS; B operand: the lane's query row, kept in
//                  registers for the whole kernel)
//   O^T += V^T P^T (A operand: V^T from LDS; B operand: P^T)
// In the transposed form a lane's 16 accumulator registers of S^T all belong to ONE query
// (column lane % 32), so the row maximum and row sum are per-lane scalars (plus one exchange
// with lane ^ 32, which holds the other half of the keys), and -- because the order of the
// contraction index inside an MFMA does not matter as long as both operands agree -- the
// exponentiated S^T registers, rounded to bf16, ARE the B operand of the second contraction:
// registers 8h..8h+7 of a lane hold keys {16h + 4g + 0..3, 16h + 8 + 4g + 0..3} (g = lane / 32),
// and the matching V^T fragment is two 8-byte LDS reads at those key offsets.  V is transposed
// on its way into LDS.  Softmax runs in fp32 with exp2 and the scale folded into one FMA.
// Tail keys are masked to -inf before the row maximum; tail query rows are clamped on load
// and not stored.  The reduction order is fixed: results are deterministic and batch-invariant.
#include "attention.h"

namespace {

constexpr int BQ = 128;
constexpr int BKV = 64;
constexpr int K_STRIDE = 72;   // bf16 per K row in LDS (64 + 8 pad: conflict-free 16-byte reads)
constexpr int V_STRIDE = 68;   // bf16 per V^T row in LDS (64 keys + 4 pad: conflict-free 8-byte reads)

__global__ __launch_bounds__(256) void attention_mfma_kernel(AttnArgs a) {
    __shared__ __attribute__((aligned(16))) bf16_t Ks[2][BKV * K_STRIDE];
    __shared__ __attribute__((aligned(16))) bf16_t Vt[2][64 * V_STRIDE];

    const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
    const int lq = lane % 32, g = lane / 32;
    const int h = blockIdx.y, b = blockIdx.z;
    const size_t bh = (size_t)b * a.heads + h;
    const int qrow = blockIdx.x * BQ + wave * 32 + lq;
    const bf16_t* qp = static_cast<const bf16_t*>(a.q) + (bh * a.n_q + min(qrow, a.n_q - 1)) * 64;
    const bf16_t* kp = static_cast<const bf16_t*>(a.k) + bh * a.n_kv * 64;
    const bf16_t* vp = static_cast<const bf16_t*>(a.v) + bh * a.n_kv * 64;

    bf16x8 qf[4];
#pragma unroll
    for (int kk = 0; kk < 4; kk++) qf[kk] = *reinterpret_cast<const bf16x8*>(qp + kk * 16 + g * 8);

    const int ld_row = tid / 8, ld_vec = tid % 8;
    bf16x8 k_reg[2], v_reg[2];
    auto load_tile = [&](int t) {
#pragma unroll
        for (int i = 0; i < 2; i++) {
            const size_t row = (size_t)min(t * BKV + ld_row + 32 * i, a.n_kv - 1);
            k_reg[i] = *reinterpret_cast<const bf16x8*>(kp + row * 64 + ld_vec * 8);
            v_reg[i] = *reinterpret_cast<const bf16x8*>(vp + row * 64 + ld_vec * 8);
        }
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 2; i++) {
            const int row = ld_row + 32 * i;
            *reinterpret_cast<bf16x8*>(&Ks[buf][row * K_STRIDE + ld_vec * 8]) = k_reg[i];
#pragma unroll
            for (int j = 0; j < 8; j++) Vt[buf][(ld_vec * 8 + j) * V_STRIDE + row] = v_reg[i][j];
        }
    };

    const float c = a.scale * 1.4426950408889634f;   // scores are exponentiated in base 2
    float m_run = -__builtin_inff(), l_run = 0.f;
    f32x16 o[2];
#pragma unroll
    for (int dt = 0; dt < 2; dt++)
#pragma unroll
        for (int i = 0; i < 16; i++) o[dt][i] = 0.f;

    const int nt = (a.n_kv + BKV - 1) / BKV;
    load_tile(0);
    store_tile(0);
    __syncthreads();
    for (int t = 0; t < nt; t++) {
        const int cur = t & 1;
        if (t + 1 < nt) load_tile(t + 1);

        f32x16 s[2];
#pragma unroll
        for (int kt = 0; kt < 2; kt++) {
#pragma unroll
            for (int i = 0; i < 16; i++) s[kt][i] = 0.f;
#pragma unroll
            for (int kk = 0; kk < 4; kk++) {
                const bf16x8 kf = *reinterpret_cast<const bf16x8*>(&Ks[cur][(kt * 32 + lq) * K_STRIDE + kk * 16 + g * 8]);
                s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], s[kt], 0, 0, 0);
            }
        }
        if (t == nt - 1 && (a.n_kv % BKV) != 0) {
#pragma unroll
            for (int kt = 0; kt < 2; kt++)
#pragma unroll
                for (int i = 0; i < 16; i++) {
                    const int key = t * BKV + kt * 32 + 8 * (i / 4) + 4 * g + (i % 4);
                    if (key >= a.n_kv) s[kt][i] = -__builtin_inff();
                }
        }
        float mx = s[0][0];
#pragma unroll
        for (int kt = 0; kt < 2; kt++)
#pragma unroll
            for (int i = 0; i < 16; i++) mx = fmaxf(mx, s[kt][i]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m_run, mx);
        const float corr = __builtin_amdgcn_exp2f((m_run - m_new) * c);
        const float mc = m_new * c;
        m_run = m_new;
        float psum = 0.f;
        bf16x8 pb[2][2];
#pragma unroll
        for (int kt = 0; kt < 2; kt++)
#pragma unroll
            for (int i = 0; i < 16; i++) {
                const float p = __builtin_amdgcn_exp2f(fmaf(s[kt][i], c, -mc));
                psum += p;
                pb[kt][i / 8][i % 8] = (bf16_t)p;
            }
        l_run = fmaf(l_run, corr, psum);
#pragma unroll
        for (int dt = 0; dt < 2; dt++)
#pragma unroll
            for (int i = 0; i < 16; i++) o[dt][i] *= corr;

#pragma unroll
        for (int dt = 0; dt < 2; dt++)
#pragma unroll
            for (int kt = 0; kt < 2; kt++)
#pragma unroll
                for (int hf = 0; hf < 2; hf++) {
                    const bf16_t* vrow = &Vt[cur][(dt * 32 + lq) * V_STRIDE + kt * 32 + hf * 16 + 4 * g];
                    const bf16x4 lo = *reinterpret_cast<const bf16x4*>(vrow);
                    const bf16x4 hi = *reinterpret_cast<const bf16x4*>(vrow + 8);
                    const bf16x8 vf = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                    o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pb[kt][hf], o[dt], 0, 0, 0);
                }

        if (t + 1 < nt) store_tile(cur ^ 1);
        __syncthreads();
    }

    if (qrow >= a.n_q) return;
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    const float inv = 1.0f / l_tot;
    const int hd = a.heads * 64;
    bf16_t* orow;
    if (qrow < a.split) orow = static_cast<bf16_t*>(a.o) + ((size_t)b * a.split + qrow) * hd;
    else orow = static_cast<bf16_t*>(a.o2) + ((size_t)b * (a.n_q - a.split) + (qrow - a.split)) * hd;
    orow += h * 64;
#pragma unroll
    for (int dt = 0; dt < 2; dt++)
#pragma unroll
        for (int gi = 0; gi < 4; gi++) {
            const int d0 = dt * 32 + 8 * gi + 4 * g;
            bf16x4 ov = {(bf16_t)(o[dt][4 * gi] * inv), (bf16_t)(o[dt][4 * gi + 1] * inv),
                         (bf16_t)(o[dt][4 * gi + 2] * inv), (bf16_t)(o[dt][4 * gi + 3] * inv)};
            *reinterpret_cast<bf16x4*>(orow + d0) = ov;
        }
}

}  // namespace

int hyb_launch_attention_mfma(const AttnArgs& a, hipStream_t st) {
    dim3 grid((a.n_q + BQ - 1) / BQ, a.heads, a.batch), block(256);
    HybTraceScope trace("attention_mfma", "flop", 4.0 * a.batch * a.heads * (double)a.n_q * a.n_kv * 64, st);
    hipLaunchKernelGGL(attention_mfma_kernel, grid, block, 0, st, a);
    return hyb_check_launch("attention_mfma");
}
