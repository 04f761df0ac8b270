/*
 * hyb.h -- C ABI of libhyb: the per-step hot path of conditional-guidance hybrid
 * parallelism for diffusion inference, for AMD MI355X (gfx950 / CDNA4).
 *
 * The paper partitions a guided denoising step by condition: the conditional and the
 * unconditional evaluation of the denoiser f_theta are the two data-parallel units
 * (Sec. 4.1), their outputs are merged by classifier-free guidance (Sec. 3), their
 * relative discrepancy drives the adaptive switching (Sec. 4.2-4.3, Eq. 1-3, Alg. 1), and
 * the scheduler advances the latent.  This library is one device's share of that step:
 * the denoiser forward of one (or both, batched) guidance branches, the CFG combine, the
 * discrepancy reduction and the Euler update.
 *
 * Conventions (all entry points):
 *  - Every pointer named in a "device" argument is caller-owned GPU memory, contiguous,
 *    row-major, 16-byte aligned.  The library never allocates, frees or retains it.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *    enqueue work; they never synchronise.  Results that are scalars (discrepancies) are
 *    written to device memory so that the call stays asynchronous.
 *  - Return value: HYB_OK or an error code; on error nothing has been enqueued (except
 *    HYB_ERR_LAUNCH, which reports a failed kernel launch).  hyb_last_error_string()
 *    gives a thread-local description of the last error.
 *  - dtype HYB_BF16: weights and GEMM/attention operands are bf16 (stored as 16-bit
 *    words), accumulation, softmax, normalisation statistics, biases, modulation vectors
 *    and the residual stream are fp32.  dtype HYB_F32: everything is fp32.
 *  - Linear weights are stored [out_features, in_features] row-major; biases are fp32.
 *  - Token tensors are token-major [batch, tokens, features].
 *  - Results are deterministic and batch-invariant: a sample's result does not depend on
 *    its batch index or on what else is in the batch (no floating-point atomics).
 */
#ifndef HYB_H
#define HYB_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    HYB_OK = 0,
    HYB_ERR_NULL = 1,       /* a required pointer is NULL */
    HYB_ERR_SHAPE = 2,      /* a size is negative, inconsistent or unsupported */
    HYB_ERR_DTYPE = 3,      /* unknown or unsupported dtype / enum value */
    HYB_ERR_ALIGN = 4,      /* a device pointer is not 16-byte aligned */
    HYB_ERR_WORKSPACE = 5,  /* workspace missing or smaller than the *_workspace_bytes query */
    HYB_ERR_LAUNCH = 6      /* the HIP runtime rejected a kernel launch */
} hyb_status;

typedef enum { HYB_F32 = 0, HYB_BF16 = 1 } hyb_dtype;

/* HYB_NORM_L1: the paper's rel-MAE (Eq. 1).  HYB_NORM_L2: the relative-L2 variant. */
typedef enum { HYB_NORM_L1 = 1, HYB_NORM_L2 = 2 } hyb_norm;

typedef enum {
    HYB_EPI_BIAS = 0,          /* out = a w^T + bias                                          */
    HYB_EPI_GELU_TANH = 1,     /* out = GELUtanh(a w^T + bias)                                */
    HYB_EPI_SILU = 2,          /* out = SiLU(a w^T + bias)                                    */
    HYB_EPI_GATE_RESIDUAL = 3, /* out(fp32) = residual + gate[row / rows_per_gate] * (a w^T + bias) */
    HYB_EPI_GEGLU = 5          /* out = (a wu^T + bias[:n]) * GELUerf(a wg^T + bias[n:]), w = [wu; wg] of 2n rows */
} hyb_epilogue;

int hyb_version(void);                       /* major * 10000 + minor * 100 + patch */
const char* hyb_last_error_string(void);     /* never NULL; valid until the next call on this thread */

/* ------------------------------------------------------------------------------------------
 * Guidance step (Sec. 3 CFG equation; Eq. 1 and its velocity form in Sec. 4.2; Alg. 1 steps
 * "M_t" and "Step Denoise"; flow ODE of Sec. 3).
 * ---------------------------------------------------------------------------------------- */

/* v_out[i] = v_u[i] + scale * (v_c[i] - v_u[i]), i < n.  `scale` = 1 + w of the paper's
 * eps_c + w (eps_c - eps_u): scale 1 returns the conditional, 0 the unconditional prediction.
 * v_c, v_u, v_out: device, n elements of `dtype`; v_out may alias v_c or v_u.  n == 0 is a no-op. */
int hyb_cfg_combine(const void* v_c, const void* v_u, void* v_out, size_t n, float scale,
                    hyb_dtype dtype, void* stream);

/* out[b] = ||v_c[b] - v_u[b]||_p / ||v_u[b]||_p over the n_per_sample elements of sample b
 * (one ratio per sample; 0/0 -> 0, x/0 -> +inf).  v_c, v_u: device [batch, n_per_sample] of
 * `dtype`; out: device float[batch]; workspace: device, at least
 * hyb_discrepancy_workspace_bytes(batch, n_per_sample) bytes, contents irrelevant.
 * Sums are accumulated in a fixed order (fp32 within a thread, fp64 across threads). */
int hyb_branch_discrepancy(const void* v_c, const void* v_u, int batch, size_t n_per_sample,
                           hyb_norm p, hyb_dtype dtype, float* out,
                           void* workspace, size_t workspace_bytes, void* stream);
size_t hyb_discrepancy_workspace_bytes(int batch, size_t n_per_sample);

/* x_out[i] = x[i] + (t_next - t) * v[i], i < n: explicit Euler step of dx/dt = v.
 * dt = t_next - t is formed once on the host in fp32, the update is one fused multiply-add.
 * x, x_out: device, `x_dtype`; v: device, `v_dtype`; x_out may alias x. */
int hyb_euler_step(const void* x, const void* v, void* x_out, size_t n, float t, float t_next,
                   hyb_dtype x_dtype, hyb_dtype v_dtype, void* stream);

/* The three calls above in ONE pass over HBM: reads v_c, v_u, x once; writes x_out (fp32),
 * optionally x_out_lowp (bf16 copy of x_out for the next denoiser call) and v_out (`v_dtype`),
 * and both discrepancies.  Layout [batch, n_per_sample]; x, x_out fp32; v_* of `v_dtype`.
 * x_out may alias x.  x_out_lowp, v_out, disc_l1, disc_l2 may each be NULL (skipped).
 * disc_l1 / disc_l2: device float[batch].  Workspace as for hyb_branch_discrepancy.
 * Generalised update: x_out = a * x + b * v with (a, b) = (1, t_next - t); see hyb_cfg_disc_affine. */
int hyb_cfg_disc_euler(const void* v_c, const void* v_u, const float* x, float* x_out,
                       void* x_out_lowp, void* v_out, int batch, size_t n_per_sample,
                       float scale, float t, float t_next, float* disc_l1, float* disc_l2,
                       hyb_dtype v_dtype, void* workspace, size_t workspace_bytes, void* stream);

/* Same pass with a generic affine scheduler update x_out = a * x + b * v_cfg (DDIM, the
 * CFG-adjusted reverse mean of Sec. 3 and Euler (a = 1, b = dt) are all of this form). */
int hyb_cfg_disc_affine(const void* v_c, const void* v_u, const float* x, float* x_out,
                        void* x_out_lowp, void* v_out, int batch, size_t n_per_sample,
                        float scale, float a, float b, float* disc_l1, float* disc_l2,
                        hyb_dtype v_dtype, void* workspace, size_t workspace_bytes, void* stream);

/* hyb_cfg_disc_euler for callers that cannot allocate device memory or hand over a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments minus the
 * workspace, same kernels, same results bit for bit; the per-workgroup partial sums go to a device array
 * built into the library (HYB_STATIC_SCRATCH_BYTES, held once per GPU for the life of the process).  The call
 * allocates and frees nothing.  Sizes whose partial sums do not fit -- hyb_discrepancy_workspace_bytes(batch,
 * n_per_sample) > HYB_STATIC_SCRATCH_BYTES, i.e. more than 32768 chunks of 256 elements over all samples --
 * are HYB_ERR_WORKSPACE (without discrepancy outputs no scratch is used and any size is accepted).  All calls
 * on one GPU share the array: calls that overlap in time on the same GPU (different streams) race on it. */
#define HYB_STATIC_SCRATCH_BYTES (1 << 20)
int hyb_cfg_disc_euler_noalloc(const void* v_c, const void* v_u, const float* x, float* x_out,
                               void* x_out_lowp, void* v_out, int batch, size_t n_per_sample,
                               float scale, float t, float t_next, float* disc_l1, float* disc_l2,
                               hyb_dtype v_dtype, void* stream);

/* ------------------------------------------------------------------------------------------
 * Denoiser f_theta(x_t, c, t) of one guidance branch (Sec. 4.1): building blocks.
 * The paper treats f_theta as a black box; the block below is the joint image+text
 * transformer block of the flow-matching model it evaluates (MMDiT layout).
 * ---------------------------------------------------------------------------------------- */

/* o = softmax(q k^T * scale) v per (batch, head).
 * q: device [batch, heads, n_q, head_dim]; k, v: device [batch, heads, n_kv, head_dim];
 * o: device [batch, n_q, heads * head_dim] (heads merged, feature = head * head_dim + i).
 * For joint attention n_q = n_kv = n_img + n_txt with image tokens first; n_q != n_kv is
 * cross-attention.  scale <= 0 means 1 / sqrt(head_dim).  head_dim must be 64.
 * n_q == 0 or batch == 0 is a no-op; n_kv == 0 with n_q > 0 is HYB_ERR_SHAPE.
 * The bf16 kernel first sums 2^(score * scale * log2 e) without a reference maximum; a workgroup (128 query rows)
 * one of whose row sums leaves [2^-64, 2^64] starts over with a running maximum, so the result is the softmax
 * for every finite input, and an input whose scaled scores exceed about +-44 takes up to twice as long. */
int hyb_joint_attention(const void* q, const void* k, const void* v, void* o,
                        int batch, int heads, int n_q, int n_kv, int head_dim, float scale,
                        hyb_dtype dtype, void* stream);

/* The same attention with a caller-provided scratch buffer.  With it the bf16 kernel may cut the query
 * blocks that would overload some compute units into parts along the keys and merge the unnormalised
 * partial results (accumulator, maximum, normaliser) in a second kernel, in a fixed order: the result is
 * deterministic, equal to hyb_joint_attention's up to the rounding of the merge, and the launch is
 * shorter (this is the form hyb_block_forward uses).  workspace: device, at least
 * hyb_joint_attention_workspace_bytes(batch, heads, n_q, dtype) bytes (0 for shapes that are never
 * split and for HYB_F32: workspace may then be NULL), contents irrelevant on entry. */
int hyb_joint_attention_ws(const void* q, const void* k, const void* v, void* o,
                           int batch, int heads, int n_q, int n_kv, int head_dim, float scale,
                           hyb_dtype dtype, void* workspace, size_t workspace_bytes, void* stream);
size_t hyb_joint_attention_workspace_bytes(int batch, int heads, int n_q, hyb_dtype dtype);

/* The same attention (workspace form) for queries that already carry the softmax scale and the change of base:
 * q holds q * scale * log2(e), so that q k^T is the exponent of 2 and o = softmax_2(q k^T) v, which is
 * softmax(q_unscaled k^T * scale) v.  A producer that rounds q to bf16 anyway (hyb_block_forward's QKV
 * projection does this) folds the factor in before its one rounding and loses nothing.  The bf16 kernel's
 * first attempt (sums without a reference maximum, see hyb_joint_attention) then needs no multiplication per
 * score either: P = 2^score; the fallback for row sums outside [2^-64, 2^64] is the same.  HYB_F32 inputs take the
 * plain fp32 kernel with scale = ln 2.  Same shapes, workspace and error behaviour as hyb_joint_attention_ws
 * (Sec. 3 of the paper: the attention inside one evaluation of the denoiser). */
int hyb_joint_attention_prescaled(const void* q, const void* k, const void* v, void* o,
                                  int batch, int heads, int n_q, int n_kv, int head_dim,
                                  hyb_dtype dtype, void* workspace, size_t workspace_bytes, void* stream);

/* out[b, r] = sum_k w[r, k] * SiLU(temb[b, k]) + bias[r]: the adaLN modulation vectors of any
 * number of blocks / streams at once (stack their weight matrices along rows).
 * w: device [rows, hidden] of `dtype`; bias: device float[rows]; temb: device float[batch, hidden];
 * out: device float[batch, rows].  hidden % 8 == 0. */
int hyb_adaln_modulation(const void* w, const float* bias, const float* temb, float* out,
                         int rows, int hidden, int batch, hyb_dtype dtype, void* stream);

/* out[b, n, :] = LN(x[b, n, :]) * (1 + scale[b, :]) + shift[b, :], LN over the feature axis with
 * biased variance and no affine.  x: device float[batch, tokens, hidden]; shift, scale: device
 * float, element (b, j) at shift[b * mod_stride + j]; out: device [batch, tokens, hidden] of
 * `out_dtype`.  shift == scale == NULL gives the plain LayerNorm.  hidden % 4 == 0, <= 8192. */
int hyb_layernorm_modulate(const float* x, const float* shift, const float* scale, size_t mod_stride,
                           void* out, int batch, int tokens, int hidden, float eps,
                           hyb_dtype out_dtype, void* stream);

/* out = epilogue(a w^T + bias).  a: device [m, k] of `dtype`; w: device [n, k] of `dtype`;
 * bias: device float[n] or NULL; out: device [m, n] of `out_dtype` (fp32 required for
 * HYB_EPI_GATE_RESIDUAL).  residual: device float[m, n] (may alias out); gate: device float,
 * element (row r, column j) at gate[(r / rows_per_gate) * gate_stride + j], or NULL for gate 1.
 * HYB_EPI_GEGLU (the gated feed-forward of the SDXL-shaped block): w is [2n, k], rows [0, n) the value half and
 * rows [n, 2n) the gate half, bias float[2n] or NULL, exact (erf) GELU on the gate.
 * k % 8 == 0 and n % 8 == 0 for bf16.  m == 0 is a no-op. */
int hyb_linear(const void* a, const void* w, const float* bias, void* out, int m, int n, int k,
               hyb_dtype dtype, hyb_dtype out_dtype, hyb_epilogue epi,
               const float* residual, const float* gate, int rows_per_gate, size_t gate_stride,
               void* stream);

typedef struct {
    int batch;        /* samples (1 = one guidance branch, 2 = conditional + unconditional) */
    int n_img;        /* image tokens per sample */
    int n_txt;        /* text tokens per sample (may be 0) */
    int hidden;       /* D = heads * head_dim */
    int heads;
    int head_dim;     /* must be 64 */
    int mlp_ratio;    /* MLP inner width = mlp_ratio * hidden */
    hyb_dtype dtype;
    float ln_eps;     /* 1e-6 for the MMDiT block */
    int txt_pre_only; /* non-zero: the text stream only supplies keys and values (see hyb_block_forward) */
} hyb_block_desc;

typedef struct {
    const void *w_qkv, *w_out, *w_fc1, *w_fc2;        /* [3D, D], [D, D], [rD, D], [D, rD] of dtype */
    const float *b_qkv, *b_out, *b_fc1, *b_fc2;       /* fp32 */
} hyb_stream_weights;

typedef struct { hyb_stream_weights img, txt; } hyb_block_weights;

/* One joint block.  For each stream s in {img, txt} with modulation vectors
 * (shift1, scale1, gate1, shift2, scale2, gate2) = the six hidden-sized chunks of mod_s[b, :]:
 *   h = LN(x_s)(1 + scale1) + shift1;  q, k, v = split3(h Wqkv^T + b), heads of 64 features
 *   o = softmax(Q K^T / 8) V over the concatenated (image first) tokens of both streams
 *   x_s += gate1 * (o_s Wout^T + b);   h2 = LN(x_s)(1 + scale2) + shift2
 *   x_s += gate2 * (GELUtanh(h2 W1^T + b1) W2^T + b2)
 * x_img_in / x_img_out: device float[batch, n_img, hidden]; x_txt_*: device float[batch, n_txt,
 * hidden]; outputs may alias inputs.  mod_img, mod_txt: device float[batch, 6 * hidden] with row
 * stride mod_stride (from hyb_adaln_modulation).  workspace: device,
 * >= hyb_block_workspace_bytes(desc) bytes.
 * desc->txt_pre_only (the last block of a model, whose text output nothing reads): the text
 * stream is modulated and projected (its keys and values enter the attention) and that is all --
 * no text queries, output projection or MLP; x_txt_out is NOT written.  The image output is the
 * same as without the flag. */
int hyb_block_forward(const hyb_block_desc* desc, const hyb_block_weights* weights,
                      const float* x_img_in, const float* x_txt_in,
                      const float* mod_img, const float* mod_txt, size_t mod_stride,
                      float* x_img_out, float* x_txt_out,
                      void* workspace, size_t workspace_bytes, void* stream);
size_t hyb_block_workspace_bytes(const hyb_block_desc* desc);

/* Sinusoidal timestep features: out[b, j] = cos(1000 t[b] f_j), out[b, dim/2 + j] = sin(1000 t[b] f_j),
 * f_j = exp(-ln(10000) j / (dim/2)).  t: device float[batch]; out: device [batch, dim] of `out_dtype`. */
int hyb_timestep_embedding(const float* t, void* out, int batch, int dim, hyb_dtype out_dtype, void* stream);

/* latent[batch, hh, ww, c] (channels last, fp32) -> tokens[batch, (hh/p)(ww/p), p*p*c] of `out_dtype`,
 * patch vector ordered (dy, dx, c); hyb_unpatchify is the inverse (tokens of `in_dtype` -> out of
 * `out_dtype`). */
int hyb_patchify(const float* latent, void* tokens, int batch, int hh, int ww, int c, int p,
                 hyb_dtype out_dtype, void* stream);
int hyb_unpatchify(const void* tokens, void* latent, int batch, int hh, int ww, int c, int p,
                   hyb_dtype in_dtype, hyb_dtype out_dtype, void* stream);

/* Element-wise conversion fp32 -> `out_dtype` (n elements), e.g. context tokens to bf16. */
int hyb_convert(const float* in, void* out, size_t n, hyb_dtype out_dtype, void* stream);

/* ------------------------------------------------------------------------------------------
 * Second denoiser shape (the U-Net family of Sec. 5's setup): one transformer block of an
 * SDXL-shaped attention stage on token-major activations.
 * ---------------------------------------------------------------------------------------- */

/* out = GroupNorm(x) * gamma + beta on x[batch, tokens, channels]: groups of channels / groups
 * consecutive channels, statistics over (tokens, channels / groups) per sample, biased variance.
 * x, out: device float (may alias); gamma, beta: device float[channels]; workspace: device,
 * >= hyb_groupnorm_workspace_bytes(batch, groups).  channels % (4 * groups) == 0, channels <= 4096. */
int hyb_groupnorm(const float* x, const float* gamma, const float* beta, float* out,
                  int batch, int tokens, int channels, int groups, float eps,
                  void* workspace, size_t workspace_bytes, void* stream);
size_t hyb_groupnorm_workspace_bytes(int batch, int groups);

/* out[r, :] = LN(x[r, :]) * gamma + beta (biased variance).  x: device float[rows, hidden];
 * gamma, beta: device float[hidden]; out: device [rows, hidden] of `out_dtype`.  hidden % 4 == 0, <= 2048. */
int hyb_layernorm_affine(const float* x, const float* gamma, const float* beta, void* out,
                         int rows, int hidden, float eps, hyb_dtype out_dtype, void* stream);

typedef struct {
    int batch;        /* samples (2 = conditional + unconditional) */
    int tokens;       /* spatial tokens per sample */
    int channels;     /* C = heads * head_dim */
    int heads;
    int head_dim;     /* must be 64 */
    int n_ctx;        /* text tokens per sample */
    int ctx_dim;      /* text feature width (multiple of 64 for bf16) */
    int groups;       /* GroupNorm groups (32) */
    hyb_dtype dtype;
    float gn_eps;     /* 1e-5 */
    float ln_eps;     /* 1e-5 */
} hyb_sdxl_block_desc;

typedef struct {
    const float *gn_g, *gn_b, *ln1_g, *ln1_b, *ln2_g, *ln2_b, *ln3_g, *ln3_b;   /* fp32 [C] */
    const void* w_qkv1;   /* [3C, C]: rows = [Wq; Wk; Wv] of the self-attention (no bias) */
    const void* w_o1;     /* [C, C] */
    const float* b_o1;
    const void* w_q2;     /* [C, C] (no bias) */
    const void* w_kv2;    /* [2C, ctx_dim]: rows = [Wk; Wv] of the cross-attention (no bias) */
    const void* w_o2;     /* [C, C] */
    const float* b_o2;
    const void* w_ff1;    /* [8C, C]: rows [0, 4C) = value half, rows [4C, 8C) = gate half */
    const float* b_ff1;   /* [8C] */
    const void* w_ff2;    /* [C, 4C] */
    const float* b_ff2;
} hyb_sdxl_block_weights;

/* g = GroupNorm(x); a = g + SelfAttn(LN(g)); b = a + CrossAttn(LN(a), ctx);
 * out = x + b + W2 (u * GELUerf(gate)) + b2 with [u, gate] = LN(b) W1^T + b1 (heads of 64 features,
 * attention scale 1/8, LayerNorms with gamma / beta).
 * x_in, x_out: device float[batch, tokens, channels] (may alias); ctx: device [batch, n_ctx, ctx_dim]
 * of desc->dtype; workspace: device, >= hyb_sdxl_block_workspace_bytes(desc). */
int hyb_sdxl_block_forward(const hyb_sdxl_block_desc* desc, const hyb_sdxl_block_weights* weights,
                           const float* x_in, const void* ctx, float* x_out,
                           void* workspace, size_t workspace_bytes, void* stream);
size_t hyb_sdxl_block_workspace_bytes(const hyb_sdxl_block_desc* desc);

/* ------------------------------------------------------------------------------------------
 * Adaptive parallelism switching (Sec. 4.3, Eq. 2-3, Alg. 1): host-side controller, no device work.
 * Steps are counted upwards in sampling order, i = 0 .. total_steps - 1.  With the discrepancy M_i
 * of step i (Eq. 1, from hyb_branch_discrepancy / hyb_cfg_disc_euler), the slope over the last
 * `window` steps is read as the rate of decline G_i = (M[i - window] - M[i]) / window; tau1 is the
 * first i >= window with 0 <= G_i < g_slope, capped by cap = min(tau_cap, total_steps - 1 - k) (and
 * set to cap when step cap is reached without the test firing); tau2 = tau1 + k.  The cap keeps
 * Eq. 3's bound 1 <= k < total_steps - tau1 for every history, so tau2 is always a step of the run;
 * k > total_steps - 1 is HYB_ERR_SHAPE.  Stage of step i: 0 = warm-up
 * (i <= tau1 or tau1 not yet known), 1 = parallelism (tau1 < i < tau2), 2 = fully-connecting.
 * The paper's settings: SDXL window 12, g_slope 0.4e-3, k 5, tau_cap 15; SD3 15, 0.1e-3, 5, 40.
 * ---------------------------------------------------------------------------------------- */
#define HYB_SWITCH_MAX_STEPS 1024
typedef struct {
    int total_steps, window, tau_cap, k;
    float g_slope;
    int step;                 /* number of discrepancies pushed so far */
    int tau1, tau2;           /* -1 until determined */
    double history[HYB_SWITCH_MAX_STEPS];
} hyb_switch_state;

/* state: HOST memory owned by the caller. */
int hyb_switch_init(hyb_switch_state* state, int total_steps, int window, float g_slope, int tau_cap, int k);
/* Record M of the next step (call once per step, in order; the value is ignored once tau1 is known);
 * *stage (may be NULL) receives the stage of that step. */
int hyb_switch_push(hyb_switch_state* state, float discrepancy, int* stage);
/* Stage of an arbitrary step under the boundaries known so far. */
int hyb_switch_stage(const hyb_switch_state* state, int step);

/* ------------------------------------------------------------------------------------------
 * Optional per-launch timing, for benchmarks (callers that measure, not the paper's method).
 * While enabled, every kernel launch of the library is bracketed by two events on its stream.
 * hyb_trace_enable(1) clears earlier records.  hyb_trace_summary waits for the recorded events
 * and writes one line per kernel: name <TAB> unit ("flop" | "byte") <TAB> launches <TAB>
 * total milliseconds <TAB> total algorithmic work.  buf: HOST memory of `cap` bytes.
 * Not thread-safe with respect to concurrent launches from other threads.
 * ---------------------------------------------------------------------------------------- */
int hyb_trace_enable(int on);
int hyb_trace_summary(char* buf, size_t cap);

#ifdef __cplusplus
}
#endif
#endif /* HYB_H */
