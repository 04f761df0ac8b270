// Bandwidth-bound pieces of the denoiser forward: LayerNorm + adaLN modulate, the adaLN
// modulation GEMV, GroupNorm, timestep features, patchify / unpatchify, dtype conversion.
// (The denoiser f_theta is a black box in the paper, Sec. 4.1; these are the parts of the
// transformer block around the contractions.)
#include "common.h"

#include <type_traits>

namespace {

// ------------------------------------------------------------------------------------------
// LayerNorm (+ modulate / affine).  One wave per row; the row lives in registers (hidden <=
// 2048), statistics are two-pass in fp32 with wavefront-shuffle reductions.
//   AFFINE = false: out = xhat * (1 + scale[b]) + shift[b]   (adaLN; shift/scale may be NULL)
//   AFFINE = true : out = xhat * scale + shift               (gamma / beta per feature)
// ------------------------------------------------------------------------------------------
constexpr int kLnMaxVec = 8;   // float4 per lane -> hidden <= 8 * 64 * 4 = 2048

// Up to two independent row sets (the image and the text stream of a joint block) share one launch:
// workgroups [0, blocks0) serve set 0, the rest set 1.
struct LnSet {
    const float* x;
    const float* shift;
    const float* scale;
    void* out;
    size_t mod_stride;
    int rows, tokens;
};
struct LnArgs {
    LnSet s[2];
    int blocks0;
    int hidden;
    float eps;
};

template <typename OT, bool AFFINE>
__global__ __launch_bounds__(256) void layernorm_kernel(LnArgs a) {
    const int wave = threadIdx.x / HYB_WAVE, lane = threadIdx.x % HYB_WAVE;
    const int blk = (int)blockIdx.x;
    const int set = blk >= a.blocks0 ? 1 : 0;
    const LnSet& p = a.s[set];
    const int row = (blk - (set ? a.blocks0 : 0)) * 4 + wave;
    if (row >= p.rows) return;
    const float* __restrict__ x = p.x;
    const float* __restrict__ shift = p.shift;
    const float* __restrict__ scale = p.scale;
    OT* __restrict__ out = static_cast<OT*>(p.out);
    const size_t mod_stride = p.mod_stride;
    const int tokens = p.tokens, hidden = a.hidden;
    const float eps = a.eps;
    const int nvec = hidden / 4;
    const f32x4* xr = reinterpret_cast<const f32x4*>(x + (size_t)row * hidden);
    f32x4 r[kLnMaxVec];
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < kLnMaxVec; i++) {
        const int c = lane + i * HYB_WAVE;
        if (c < nvec) {
            r[i] = xr[c];
            s += (r[i][0] + r[i][1]) + (r[i][2] + r[i][3]);
        }
    }
    const float mean = wave_sum(s) / (float)hidden;
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < kLnMaxVec; i++) {
        const int c = lane + i * HYB_WAVE;
        if (c < nvec) {
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const float d = r[i][j] - mean;
                q = fmaf(d, d, q);
            }
        }
    }
    const float rstd = rsqrtf(wave_sum(q) / (float)hidden + eps);
    const size_t b = (size_t)(row / tokens);
    const f32x4* sh = shift ? reinterpret_cast<const f32x4*>(shift + (AFFINE ? 0 : b * mod_stride)) : nullptr;
    const f32x4* sc = scale ? reinterpret_cast<const f32x4*>(scale + (AFFINE ? 0 : b * mod_stride)) : nullptr;
    OT* orow = out + (size_t)row * hidden;
#pragma unroll
    for (int i = 0; i < kLnMaxVec; i++) {
        const int c = lane + i * HYB_WAVE;
        if (c < nvec) {
            f32x4 y;
            const f32x4 a = sc ? sc[c] : (f32x4){0.f, 0.f, 0.f, 0.f};
            const f32x4 bb = sh ? sh[c] : (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const float xh = (r[i][j] - mean) * rstd;
                const float g = AFFINE ? (sc ? a[j] : 1.f) : 1.f + a[j];
                y[j] = fmaf(xh, g, bb[j]);
            }
            if constexpr (sizeof(OT) == 4) {
                *reinterpret_cast<f32x4*>(orow + 4 * c) = y;
            } else {
                bf16x4 o = {(bf16_t)y[0], (bf16_t)y[1], (bf16_t)y[2], (bf16_t)y[3]};
                *reinterpret_cast<bf16x4*>(orow + 4 * c) = o;
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// adaLN modulation GEMV: out[b, r] = sum_k w[r, k] SiLU(temb[b, k]) + bias[r].  Weight-read bound:
// one wave per row streams the row with 16-byte loads; SiLU(temb) of up to kAdaMaxBatch samples
// sits in LDS.
// ------------------------------------------------------------------------------------------
constexpr int kAdaMaxBatch = 4;
constexpr int kAdaRowsPerWave = 4;

// (the weights are streamed once per call: non-temporal loads, which do not displace what the caches hold)
template <typename WT> __device__ __forceinline__ void load8(const WT* p, float* r);
template <> __device__ __forceinline__ void load8<float>(const float* p, float* r) {
    const f32x4 a = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
    const f32x4 b = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p + 4));
    r[0] = a[0]; r[1] = a[1]; r[2] = a[2]; r[3] = a[3]; r[4] = b[0]; r[5] = b[1]; r[6] = b[2]; r[7] = b[3];
}
template <> __device__ __forceinline__ void load8<bf16_t>(const bf16_t* p, float* r) {
    const u32x4 a = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));   // bf16 -> fp32: the bits, shifted up
#pragma unroll
    for (int i = 0; i < 4; i++) {
        r[2 * i] = __uint_as_float(a[i] << 16);
        r[2 * i + 1] = __uint_as_float(a[i] & 0xffff0000u);
    }
}

template <typename WT>
__global__ __launch_bounds__(256) void adaln_kernel(const WT* __restrict__ w, const float* __restrict__ bias,
                                                    const float* __restrict__ temb, float* __restrict__ out, int rows,
                                                    int hidden, int batch, int out_stride) {
    extern __shared__ float s_act[];   // [batch][hidden]
    for (int i = threadIdx.x; i < batch * hidden; i += blockDim.x) s_act[i] = silu_f(temb[i]);
    __syncthreads();
    const int wave = threadIdx.x / HYB_WAVE, lane = threadIdx.x % HYB_WAVE;
    const int row0 = (blockIdx.x * 4 + wave) * kAdaRowsPerWave;
    float acc[kAdaRowsPerWave][kAdaMaxBatch];
#pragma unroll
    for (int r = 0; r < kAdaRowsPerWave; r++)
#pragma unroll
        for (int b = 0; b < kAdaMaxBatch; b++) acc[r][b] = 0.f;
    for (int k = lane * 8; k < hidden; k += HYB_WAVE * 8) {
        float wv[kAdaRowsPerWave][8];
#pragma unroll
        for (int r = 0; r < kAdaRowsPerWave; r++) {
            const int row = min(row0 + r, rows - 1);
            load8<WT>(w + (size_t)row * hidden + k, wv[r]);
        }
#pragma unroll
        for (int b = 0; b < kAdaMaxBatch; b++) {
            if (b < batch) {
                const float* a = s_act + b * hidden + k;
#pragma unroll
                for (int r = 0; r < kAdaRowsPerWave; r++)
#pragma unroll
                    for (int j = 0; j < 8; j++) acc[r][b] = fmaf(wv[r][j], a[j], acc[r][b]);
            }
        }
    }
#pragma unroll
    for (int r = 0; r < kAdaRowsPerWave; r++)
#pragma unroll
        for (int b = 0; b < kAdaMaxBatch; b++) {
            const float t = wave_sum(acc[r][b]);
            if (lane == 0 && b < batch && row0 + r < rows) out[(size_t)b * out_stride + row0 + r] = t + bias[row0 + r];
        }
}

// ------------------------------------------------------------------------------------------
// GroupNorm on token-major data x[B, T, C], groups of C/G consecutive channels, statistics over
// (T, C/G) per sample.  Three kernels; 1 and 3 use one thread per 4-channel vector (so every load and
// store is a coalesced 16-byte access and a thread stays inside one group) and chunks of a few tokens, so
// that a launch has thousands of workgroups with all their loads in flight at once:
//  1. each workgroup sums x and x^2 over its chunk of tokens (fp32 per thread, then the threads of a
//     group are added in a fixed order in fp64) -> partial[b][chunk][group][2];
//  2. one workgroup per sample adds the partials (fp64; a few interleaved partial sums per group, each in
//     chunk order, then those in lane order) and forms mean and 1/std per group;
//  3. each workgroup normalises its chunk: y = (x - mean) rstd gamma + beta.
// No atomics: the result is deterministic and independent of the batch index.
// ------------------------------------------------------------------------------------------
constexpr int kGnChunks = 1024;   // at most this many chunks per sample
constexpr int kGnTokens = 4;      // tokens per chunk (more when a sample has more than kGnChunks * kGnTokens tokens)

__global__ void groupnorm_stats_kernel(const float* __restrict__ x, double* __restrict__ partial, int tokens,
                                       int channels, int groups, int tokens_per_chunk) {
    extern __shared__ float gn_red[];   // [nvec][2]
    const int nvec = channels / 4, vec = threadIdx.x;
    const int chunk = blockIdx.x, b = blockIdx.y;
    const int t0 = chunk * tokens_per_chunk, t1 = min(tokens, t0 + tokens_per_chunk);
    const f32x4* xb = reinterpret_cast<const f32x4*>(x + (size_t)b * tokens * channels);
    float s = 0.f, q = 0.f;
    for (int t = t0; t < t1; t += kGnTokens) {
        f32x4 v[kGnTokens];
#pragma unroll
        for (int j = 0; j < kGnTokens; j++) v[j] = xb[(size_t)min(t + j, t1 - 1) * nvec + vec];   // clamped: in bounds
#pragma unroll
        for (int j = 0; j < kGnTokens; j++) {
            if (t + j < t1) {
                s += (v[j][0] + v[j][1]) + (v[j][2] + v[j][3]);
                q = fmaf(v[j][0], v[j][0], q); q = fmaf(v[j][1], v[j][1], q);
                q = fmaf(v[j][2], v[j][2], q); q = fmaf(v[j][3], v[j][3], q);
            }
        }
    }
    gn_red[2 * vec] = s;
    gn_red[2 * vec + 1] = q;
    __syncthreads();
    if (vec < groups) {
        const int vpg = nvec / groups;
        double ds = 0.0, dq = 0.0;
        for (int i = 0; i < vpg; i++) {
            ds += (double)gn_red[2 * (vec * vpg + i)];
            dq += (double)gn_red[2 * (vec * vpg + i) + 1];
        }
        double* o = partial + (((size_t)b * gridDim.x + chunk) * groups + vec) * 2;
        o[0] = ds;
        o[1] = dq;
    }
}

// One workgroup per sample, `lanes` threads per group, thread = j * groups + g so that the threads of a wave
// read consecutive (sum, sum of squares) pairs: thread (g, j) adds the partials of chunks j, j + lanes, ... in
// that order (fp64), thread (g, 0) then adds the `lanes` sums in lane order and leaves (mean, 1/std) as two
// floats per group.  blockDim.x = groups * lanes.
__global__ void groupnorm_finalize_kernel(const double* __restrict__ partial, float* __restrict__ stats, int nchunks,
                                          int groups, int lanes, double count, float eps) {
    typedef double f64x2 __attribute__((ext_vector_type(2)));
    extern __shared__ double gn_fin[];   // [lanes][groups][2]
    const int g = threadIdx.x % groups, j = threadIdx.x / groups, b = blockIdx.x;
    const f64x2* p = reinterpret_cast<const f64x2*>(partial) + (size_t)b * nchunks * groups + g;
    double ds = 0.0, dq = 0.0;
    for (int c0 = j; c0 < nchunks; c0 += 8 * lanes) {     // eight loads in flight, added in chunk order
        f64x2 v[8];
#pragma unroll
        for (int u = 0; u < 8; u++) v[u] = p[(size_t)min(c0 + u * lanes, nchunks - 1) * groups];   // clamped: in bounds
#pragma unroll
        for (int u = 0; u < 8; u++)
            if (c0 + u * lanes < nchunks) { ds += v[u][0]; dq += v[u][1]; }
    }
    gn_fin[(j * groups + g) * 2] = ds;
    gn_fin[(j * groups + g) * 2 + 1] = dq;
    __syncthreads();
    if (j != 0) return;
    ds = 0.0; dq = 0.0;
    for (int i = 0; i < lanes; i++) {
        ds += gn_fin[(i * groups + g) * 2];
        dq += gn_fin[(i * groups + g) * 2 + 1];
    }
    const double mean_d = ds / count;
    const double var_d = fmax(dq / count - mean_d * mean_d, 0.0);
    stats[((size_t)b * groups + g) * 2] = (float)mean_d;
    stats[((size_t)b * groups + g) * 2 + 1] = (float)(1.0 / sqrt(var_d + (double)eps));
}

__global__ void groupnorm_apply_kernel(const float* __restrict__ x, const float* __restrict__ stats,
                                       const float* __restrict__ gamma, const float* __restrict__ beta,
                                       float* __restrict__ out, int tokens, int channels, int groups,
                                       int tokens_per_chunk) {
    const int nvec = channels / 4, vec = threadIdx.x;
    const int chunk = blockIdx.x, b = blockIdx.y;
    const int grp = vec / (nvec / groups);
    const float mean = stats[((size_t)b * groups + grp) * 2], rstd = stats[((size_t)b * groups + grp) * 2 + 1];
    const f32x4 gm = reinterpret_cast<const f32x4*>(gamma)[vec], bt = reinterpret_cast<const f32x4*>(beta)[vec];
    const f32x4* xb = reinterpret_cast<const f32x4*>(x + (size_t)b * tokens * channels);
    f32x4* ob = reinterpret_cast<f32x4*>(out + (size_t)b * tokens * channels);
    const int t0 = chunk * tokens_per_chunk, t1 = min(tokens, t0 + tokens_per_chunk);
    for (int t = t0; t < t1; t += kGnTokens) {
        f32x4 v[kGnTokens];
#pragma unroll
        for (int j = 0; j < kGnTokens; j++) v[j] = xb[(size_t)min(t + j, t1 - 1) * nvec + vec];   // clamped: in bounds
#pragma unroll
        for (int j = 0; j < kGnTokens; j++) {
            if (t + j < t1) {
                f32x4 y;
#pragma unroll
                for (int e = 0; e < 4; e++) y[e] = fmaf((v[j][e] - mean) * rstd, gm[e], bt[e]);
                ob[(size_t)(t + j) * nvec + vec] = y;
            }
        }
    }
}

template <typename OT>
__global__ void timestep_embedding_kernel(const float* t, OT* out, int batch, int dim) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= batch * dim) return;
    const int b = i / dim, j = i % dim, half = dim / 2;
    const int f = j < half ? j : j - half;
    const double ang = 1000.0 * (double)t[b] * exp(-9.210340371976184 * (double)f / (double)half);  // ln(10000)
    out[i] = from_f32<OT>((float)(j < half ? cos(ang) : sin(ang)));
}

// tokens[b, py*(ww/p)+px, (dy*p+dx)*c + ch] = latent[b, py*p+dy, px*p+dx, ch]
template <typename TT, typename LT, bool TO_TOKENS>
__global__ void patch_kernel(LT* latent, TT* tokens, int batch, int hh, int ww, int c, int p) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t total = (size_t)batch * hh * ww * c;
    if (i >= total) return;
    const int ch = i % c;
    size_t r = i / c;
    const int xw = r % ww; r /= ww;
    const int yh = r % hh;
    const size_t b = r / hh;
    const int py = yh / p, dy = yh % p, px = xw / p, dx = xw % p;
    const size_t tok = (b * (hh / p) + py) * (ww / p) + px;
    const size_t ti = tok * ((size_t)p * p * c) + (size_t)(dy * p + dx) * c + ch;
    using TV = std::remove_const_t<TT>;
    using LV = std::remove_const_t<LT>;
    if constexpr (TO_TOKENS) tokens[ti] = from_f32<TV>(to_f32<LV>(latent[i]));
    else latent[i] = from_f32<LV>(to_f32<TV>(tokens[ti]));
}

template <typename OT>
__global__ void convert_kernel(const float* in, OT* out, size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = from_f32<OT>(in[i]);
}

}  // namespace

namespace {
int launch_layernorm(const LnArgs& a, int blocks, double rows, hyb_dtype out_dtype, bool affine, hipStream_t st) {
    dim3 grid(blocks), block(256);
    HybTraceScope trace("layernorm", "byte", rows * a.hidden * (4 + hyb_dtype_size(out_dtype)), st);
    if (out_dtype == HYB_F32) {
        if (affine) hipLaunchKernelGGL((layernorm_kernel<float, true>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((layernorm_kernel<float, false>), grid, block, 0, st, a);
    } else {
        if (affine) hipLaunchKernelGGL((layernorm_kernel<bf16_t, true>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((layernorm_kernel<bf16_t, false>), grid, block, 0, st, a);
    }
    return hyb_check_launch("layernorm");
}
}  // namespace

// Internal launcher shared with the block composition (affine = gamma/beta LayerNorm).
int hyb_launch_layernorm(const float* x, const float* shift, const float* scale, size_t mod_stride, void* out,
                         int batch, int tokens, int hidden, float eps, hyb_dtype out_dtype, bool affine,
                         hipStream_t st) {
    const int rows = batch * tokens;
    if (rows == 0) return HYB_OK;
    LnArgs a{};
    a.s[0] = LnSet{x, shift, scale, out, mod_stride, rows, tokens};
    a.blocks0 = (rows + 3) / 4;
    a.hidden = hidden;
    a.eps = eps;
    return launch_layernorm(a, a.blocks0, rows, out_dtype, affine, st);
}

// Two modulated LayerNorms (no affine) of the same width in one launch; either set may be empty.
int hyb_launch_layernorm_pair(const float* const x[2], const float* const shift[2], const float* const scale[2],
                              size_t mod_stride, void* const out[2], int batch, const int tokens[2], int hidden,
                              float eps, hyb_dtype out_dtype, hipStream_t st) {
    LnArgs a{};
    int blocks[2];
    for (int i = 0; i < 2; i++) {
        const int rows = batch * tokens[i];
        a.s[i] = LnSet{x[i], shift[i], scale[i], out[i], mod_stride, rows, tokens[i] > 0 ? tokens[i] : 1};
        blocks[i] = (rows + 3) / 4;
    }
    if (blocks[0] + blocks[1] == 0) return HYB_OK;
    a.blocks0 = blocks[0];
    a.hidden = hidden;
    a.eps = eps;
    return launch_layernorm(a, blocks[0] + blocks[1], (double)batch * (tokens[0] + tokens[1]), out_dtype, false, st);
}

// chunk partials (fp64 sum and sum of squares), then (mean, 1/std) per (sample, group)
static size_t gn_partial_bytes(int batch, int groups) {
    return hyb_align_up((size_t)batch * kGnChunks * groups * 2 * sizeof(double), 256);
}
size_t hyb_groupnorm_scratch_bytes(int batch, int groups) {
    return gn_partial_bytes(batch, groups) + hyb_align_up((size_t)batch * groups * 2 * sizeof(float), 256);
}

// channels % (4 * groups) == 0 and channels <= 4096 (one thread per 4-channel vector, <= 1024 threads).
int hyb_launch_groupnorm(const float* x, const float* gamma, const float* beta, float* out, int batch, int tokens,
                         int channels, int groups, float eps, void* scratch, hipStream_t st) {
    if (batch == 0 || tokens == 0) return HYB_OK;
    HYB_REQUIRE(channels % (4 * groups) == 0 && channels <= 4096 && groups <= channels / 4, HYB_ERR_SHAPE,
                "groupnorm: channels %d must be a multiple of 4 * groups (%d) and at most 4096", channels, groups);
    const int nvec = channels / 4;
    const int want = (tokens + kGnTokens - 1) / kGnTokens;
    const int nchunks = want < kGnChunks ? want : kGnChunks;
    const int tpc = (tokens + nchunks - 1) / nchunks;
    const int used = (tokens + tpc - 1) / tpc;     // chunks that actually hold tokens (<= kGnChunks)
    dim3 grid(used, batch), block(nvec);
    HybTraceScope trace("groupnorm", "byte", (double)batch * tokens * channels * 12, st);
    hipLaunchKernelGGL(groupnorm_stats_kernel, grid, block, nvec * 2 * sizeof(float), st, x, (double*)scratch, tokens, channels, groups, tpc);
    float* stats = reinterpret_cast<float*>(static_cast<char*>(scratch) + gn_partial_bytes(batch, groups));
    int lanes = 32;                                   // groups * lanes <= 1024 threads
    while (groups * lanes > 1024) lanes /= 2;
    hipLaunchKernelGGL(groupnorm_finalize_kernel, dim3(batch), dim3(groups * lanes), groups * lanes * 2 * sizeof(double), st,
                       (const double*)scratch, stats, used, groups, lanes, (double)tokens * (channels / groups), eps);
    hipLaunchKernelGGL(groupnorm_apply_kernel, grid, block, 0, st, x, (const float*)stats, gamma, beta, out, tokens, channels, groups, tpc);
    return hyb_check_launch("groupnorm");
}

extern "C" int hyb_layernorm_modulate(const float* x, const float* shift, const float* scale, size_t mod_stride,
                                      void* out, int batch, int tokens, int hidden, float eps,
                                      hyb_dtype out_dtype, void* stream) {
    HYB_CHECK_DTYPE(out_dtype);
    HYB_REQUIRE(batch >= 0 && tokens >= 0, HYB_ERR_SHAPE, "hyb_layernorm_modulate: negative size");
    HYB_REQUIRE(hidden > 0 && hidden % 4 == 0 && hidden <= kLnMaxVec * 256, HYB_ERR_SHAPE,
                "hyb_layernorm_modulate: hidden %d must be a positive multiple of 4, at most %d", hidden, kLnMaxVec * 256);
    if (batch == 0 || tokens == 0) return HYB_OK;
    HYB_CHECK_PTR(x); HYB_CHECK_PTR(out);
    HYB_CHECK_ALIGN(x); HYB_CHECK_ALIGN(out); HYB_CHECK_ALIGN(shift); HYB_CHECK_ALIGN(scale);
    HYB_REQUIRE((shift == nullptr) == (scale == nullptr), HYB_ERR_NULL, "hyb_layernorm_modulate: shift and scale must both be given or both be NULL");
    HYB_REQUIRE(mod_stride % 4 == 0, HYB_ERR_ALIGN, "hyb_layernorm_modulate: mod_stride must be a multiple of 4");
    return hyb_launch_layernorm(x, shift, scale, mod_stride, out, batch, tokens, hidden, eps, out_dtype, false, (hipStream_t)stream);
}

extern "C" int hyb_adaln_modulation(const void* w, const float* bias, const float* temb, float* out,
                                    int rows, int hidden, int batch, hyb_dtype dtype, void* stream) {
    HYB_CHECK_DTYPE(dtype);
    HYB_REQUIRE(rows >= 0 && batch >= 0, HYB_ERR_SHAPE, "hyb_adaln_modulation: negative size");
    HYB_REQUIRE(hidden > 0 && hidden % 8 == 0 && hidden <= 4096, HYB_ERR_SHAPE,
                "hyb_adaln_modulation: hidden %d must be a positive multiple of 8, at most 4096", hidden);
    if (rows == 0 || batch == 0) return HYB_OK;
    HYB_CHECK_PTR(w); HYB_CHECK_PTR(bias); HYB_CHECK_PTR(temb); HYB_CHECK_PTR(out);
    HYB_CHECK_ALIGN(w); HYB_CHECK_ALIGN(bias); HYB_CHECK_ALIGN(temb); HYB_CHECK_ALIGN(out);
    hipStream_t st = (hipStream_t)stream;
    const int rows_per_block = 4 * kAdaRowsPerWave;
    dim3 grid((rows + rows_per_block - 1) / rows_per_block), block(256);
    HybTraceScope trace("adaln_modulation", "byte", (double)rows * hidden * hyb_dtype_size(dtype) * ((batch + kAdaMaxBatch - 1) / kAdaMaxBatch), st);
    for (int b0 = 0; b0 < batch; b0 += kAdaMaxBatch) {
        const int nb = batch - b0 < kAdaMaxBatch ? batch - b0 : kAdaMaxBatch;
        const size_t shmem = (size_t)nb * hidden * sizeof(float);
        const float* tp = temb + (size_t)b0 * hidden;
        float* op = out + (size_t)b0 * rows;
        if (dtype == HYB_BF16) hipLaunchKernelGGL((adaln_kernel<bf16_t>), grid, block, shmem, st, (const bf16_t*)w, bias, tp, op, rows, hidden, nb, rows);
        else hipLaunchKernelGGL((adaln_kernel<float>), grid, block, shmem, st, (const float*)w, bias, tp, op, rows, hidden, nb, rows);
        int rc = hyb_check_launch("hyb_adaln_modulation");
        if (rc != HYB_OK) return rc;
    }
    return HYB_OK;
}

extern "C" int hyb_timestep_embedding(const float* t, void* out, int batch, int dim, hyb_dtype out_dtype, void* stream) {
    HYB_CHECK_DTYPE(out_dtype);
    HYB_REQUIRE(batch >= 0 && dim > 0 && dim % 2 == 0, HYB_ERR_SHAPE, "hyb_timestep_embedding: batch >= 0 and an even dim > 0 required");
    if (batch == 0) return HYB_OK;
    HYB_CHECK_PTR(t); HYB_CHECK_PTR(out);
    const int n = batch * dim;
    if (out_dtype == HYB_F32) hipLaunchKernelGGL((timestep_embedding_kernel<float>), dim3((n + 255) / 256), dim3(256), 0, (hipStream_t)stream, t, (float*)out, batch, dim);
    else hipLaunchKernelGGL((timestep_embedding_kernel<bf16_t>), dim3((n + 255) / 256), dim3(256), 0, (hipStream_t)stream, t, (bf16_t*)out, batch, dim);
    return hyb_check_launch("hyb_timestep_embedding");
}

static int check_patch(const char* who, int batch, int hh, int ww, int c, int p) {
    HYB_REQUIRE(batch >= 0 && hh >= 0 && ww >= 0 && c > 0 && p > 0, HYB_ERR_SHAPE, "%s: bad sizes", who);
    HYB_REQUIRE(hh % p == 0 && ww % p == 0, HYB_ERR_SHAPE, "%s: latent %dx%d is not a multiple of patch %d", who, hh, ww, p);
    return HYB_OK;
}

extern "C" int hyb_patchify(const float* latent, void* tokens, int batch, int hh, int ww, int c, int p,
                            hyb_dtype out_dtype, void* stream) {
    HYB_CHECK_DTYPE(out_dtype);
    int rc = check_patch("hyb_patchify", batch, hh, ww, c, p);
    if (rc) return rc;
    const size_t n = (size_t)batch * hh * ww * c;
    if (n == 0) return HYB_OK;
    HYB_CHECK_PTR(latent); HYB_CHECK_PTR(tokens);
    dim3 grid((unsigned)((n + 255) / 256)), block(256);
    if (out_dtype == HYB_F32) hipLaunchKernelGGL((patch_kernel<float, const float, true>), grid, block, 0, (hipStream_t)stream, latent, (float*)tokens, batch, hh, ww, c, p);
    else hipLaunchKernelGGL((patch_kernel<bf16_t, const float, true>), grid, block, 0, (hipStream_t)stream, latent, (bf16_t*)tokens, batch, hh, ww, c, p);
    return hyb_check_launch("hyb_patchify");
}

extern "C" int hyb_unpatchify(const void* tokens, void* latent, int batch, int hh, int ww, int c, int p,
                              hyb_dtype in_dtype, hyb_dtype out_dtype, void* stream) {
    HYB_CHECK_DTYPE(in_dtype); HYB_CHECK_DTYPE(out_dtype);
    int rc = check_patch("hyb_unpatchify", batch, hh, ww, c, p);
    if (rc) return rc;
    const size_t n = (size_t)batch * hh * ww * c;
    if (n == 0) return HYB_OK;
    HYB_CHECK_PTR(latent); HYB_CHECK_PTR(tokens);
    dim3 grid((unsigned)((n + 255) / 256)), block(256);
    hipStream_t st = (hipStream_t)stream;
    if (in_dtype == HYB_F32 && out_dtype == HYB_F32) hipLaunchKernelGGL((patch_kernel<const float, float, false>), grid, block, 0, st, (float*)latent, (const float*)tokens, batch, hh, ww, c, p);
    else if (in_dtype == HYB_F32) hipLaunchKernelGGL((patch_kernel<const float, bf16_t, false>), grid, block, 0, st, (bf16_t*)latent, (const float*)tokens, batch, hh, ww, c, p);
    else if (out_dtype == HYB_F32) hipLaunchKernelGGL((patch_kernel<const bf16_t, float, false>), grid, block, 0, st, (float*)latent, (const bf16_t*)tokens, batch, hh, ww, c, p);
    else hipLaunchKernelGGL((patch_kernel<const bf16_t, bf16_t, false>), grid, block, 0, st, (bf16_t*)latent, (const bf16_t*)tokens, batch, hh, ww, c, p);
    return hyb_check_launch("hyb_unpatchify");
}

extern "C" int hyb_convert(const float* in, void* out, size_t n, hyb_dtype out_dtype, void* stream) {
    HYB_CHECK_DTYPE(out_dtype);
    if (n == 0) return HYB_OK;
    HYB_CHECK_PTR(in); HYB_CHECK_PTR(out);
    dim3 grid((unsigned)((n + 255) / 256)), block(256);
    if (out_dtype == HYB_F32) hipLaunchKernelGGL((convert_kernel<float>), grid, block, 0, (hipStream_t)stream, in, (float*)out, n);
    else hipLaunchKernelGGL((convert_kernel<bf16_t>), grid, block, 0, (hipStream_t)stream, in, (bf16_t*)out, n);
    return hyb_check_launch("hyb_convert");
}
