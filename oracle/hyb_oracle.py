"""CPU oracle for the guidance-branch hot path (TEST INFRASTRUCTURE, not product code).

Plain, slow, fp64 numpy statement of what the HIP library computes: the per-step
denoiser forward of one classifier-free-guidance branch (MMDiT joint blocks, and an
SDXL-shaped transformer stage block), the CFG combine, the cond/uncond denoising
discrepancy, the flow-matching Euler update, the shifted sigma schedule and the
adaptive switching rule.  Nothing here is blocked, fused or reordered: every function
is the textbook definition, so it can be checked against the paper by eye.

Only tests, the smoke check and the bench's cpu_baseline leg may import this module.
It shares no code with the HIP path and never imports the product package.

Where the paper fixes the math it is cited (section / equation / algorithm).  The paper
treats the denoiser f_theta as a black box (Sec. 4.1), so the block internals follow the
published MMDiT / SDXL-transformer layouts as fixed by the workload configs; those
parts are marked "parity unpinned by the paper" (pinned instead by library special
cases, brute force and invariants in the CPU tests).

Pins (tests/test_oracle_*.py): torch CPU fp64 library routines (layer_norm, group_norm,
gelu, silu, scaled_dot_product_attention; the modulated final layer re-assembled from layer_norm + linear),
pure-Python brute force on tiny inputs,
closed forms (CFG s=0/1, discrepancy of scaled branches, Euler telescoping, sigma
closed form, constant velocity through the whole sampling loop) and structural invariants
(zero modulation => identity block, key permutation invariance, softmax rows sum to one,
a guidance branch with zero weight does not matter).
"""
import math

import numpy as np
from scipy.special import erf as _erf

F64 = np.float64


def _f64(a):
    return np.asarray(a, dtype=F64)


# --------------------------------------------------------------------------------------
# Elementwise functions
# --------------------------------------------------------------------------------------
def silu(z):
    """SiLU(z) = z * sigmoid(z)."""
    z = _f64(z)
    return z / (1.0 + np.exp(-z))


def gelu_tanh(z):
    """GELU, tanh form: 0.5 z (1 + tanh(sqrt(2/pi) (z + 0.044715 z^3)))."""
    z = _f64(z)
    return 0.5 * z * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (z + 0.044715 * z ** 3)))


def gelu_erf(z):
    """GELU, exact form: 0.5 z (1 + erf(z / sqrt 2))."""
    z = _f64(z)
    return 0.5 * z * (1.0 + _erf(z / math.sqrt(2.0)))


# --------------------------------------------------------------------------------------
# Normalisations and linear maps
# --------------------------------------------------------------------------------------
def layer_norm(x, eps=1e-6):
    """LayerNorm over the last axis, biased variance, no affine."""
    x = _f64(x)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps)


def layer_norm_affine(x, gamma, beta, eps=1e-5):
    """LayerNorm over the last axis followed by gamma * xhat + beta."""
    return layer_norm(x, eps) * _f64(gamma) + _f64(beta)


def group_norm(x, groups, gamma, beta, eps=1e-5):
    """GroupNorm on token-major data x[B, T, C]: channels are split into `groups` runs of
    C/groups consecutive channels; statistics are taken over (T, C/groups) per sample."""
    x = _f64(x)
    B, T, C = x.shape
    cg = C // groups
    xg = x.reshape(B, T, groups, cg)
    mu = xg.mean(axis=(1, 3), keepdims=True)
    var = ((xg - mu) ** 2).mean(axis=(1, 3), keepdims=True)
    xh = ((xg - mu) / np.sqrt(var + eps)).reshape(B, T, C)
    return xh * _f64(gamma) + _f64(beta)


def linear(x, W, b=None):
    """y = x W^T (+ b), W stored [out, in]."""
    y = _f64(x) @ _f64(W).T
    if b is not None:
        y = y + _f64(b)
    return y


def modulate(xhat, shift, scale):
    """adaLN modulation: xhat * (1 + scale) + shift, shift/scale broadcast over tokens."""
    return xhat * (1.0 + scale[:, None, :]) + shift[:, None, :]


# --------------------------------------------------------------------------------------
# Embeddings
# --------------------------------------------------------------------------------------
def timestep_embedding(t, dim=256):
    """Sinusoidal embedding of tau = 1000 t: [cos(tau f_j), sin(tau f_j)], j < dim/2,
    f_j = exp(-ln(10000) j / (dim/2)).  t: [B] -> [B, dim]."""
    t = _f64(t).reshape(-1)
    half = dim // 2
    f = np.exp(-math.log(10000.0) * np.arange(half, dtype=F64) / half)
    ang = (1000.0 * t)[:, None] * f[None, :]
    return np.concatenate([np.cos(ang), np.sin(ang)], axis=1)


def timestep_mlp(t, w1, b1, w2, b2, dim=256):
    """temb = W2 SiLU(W1 sincos(1000 t) + b1) + b2."""
    return linear(silu(linear(timestep_embedding(t, dim), w1, b1)), w2, b2)


def patchify(latent, p):
    """latent[B, Hh, Ww, C] (channels last) -> tokens[B, (Hh/p)(Ww/p), p*p*C]; the patch
    vector is ordered (dy, dx, c); tokens are row-major over the patch grid."""
    x = _f64(latent)
    B, Hh, Ww, C = x.shape
    x = x.reshape(B, Hh // p, p, Ww // p, p, C).transpose(0, 1, 3, 2, 4, 5)
    return x.reshape(B, (Hh // p) * (Ww // p), p * p * C)


def unpatchify(tokens, Hh, Ww, C, p):
    """Inverse of patchify."""
    x = _f64(tokens)
    B = x.shape[0]
    x = x.reshape(B, Hh // p, Ww // p, p, p, C).transpose(0, 1, 3, 2, 4, 5)
    return x.reshape(B, Hh, Ww, C)


# --------------------------------------------------------------------------------------
# Attention
# --------------------------------------------------------------------------------------
def softmax_rows(S):
    """Row softmax with the row maximum subtracted."""
    S = _f64(S)
    P = np.exp(S - S.max(axis=-1, keepdims=True))
    return P / P.sum(axis=-1, keepdims=True)


def attention(q, k, v, scale=None, rows=None, chunk=1024):
    """softmax(q k^T * scale) v per (batch, head).

    q[B, H, Nq, d], k, v[B, H, Nk, d] -> o[B, Nq, H*d] (heads merged, feature = head*d+i).
    scale defaults to 1/sqrt(d).  `rows` (optional index array) restricts the computation
    to those query rows (output [B, len(rows), H*d]); the score matrix is formed `chunk`
    query rows at a time only to bound memory, each row is still the plain definition."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    B, H, Nq, d = q.shape
    if scale is None or scale <= 0:
        scale = 1.0 / math.sqrt(d)
    if rows is not None:
        q = q[:, :, np.asarray(rows), :]
        Nq = q.shape[2]
    o = np.empty((B, Nq, H * d), dtype=F64)
    for b in range(B):
        for h in range(H):
            for r0 in range(0, Nq, chunk):
                S = (q[b, h, r0:r0 + chunk] @ k[b, h].T) * scale
                o[b, r0:r0 + chunk, h * d:(h + 1) * d] = softmax_rows(S) @ v[b, h]
    return o


def split_heads(y, H):
    """y[B, N, H*d] -> [B, H, N, d] (feature index = head*d + i)."""
    B, N, HD = y.shape
    return y.reshape(B, N, H, HD // H).transpose(0, 2, 1, 3)


# --------------------------------------------------------------------------------------
# MMDiT joint block and branch forward (block internals: parity unpinned by the paper;
# the paper only fixes the outer contract f_theta(x_t, c, t), Sec. 4.1)
# --------------------------------------------------------------------------------------
def adaln_modulation(temb, ada_w, ada_b, chunks=6):
    """mod = W_ada SiLU(temb) + b_ada, split into `chunks` equal parts along features.
    For a joint block the order is (shift1, scale1, gate1, shift2, scale2, gate2)."""
    mod = linear(silu(temb), ada_w, ada_b)
    return np.split(mod, chunks, axis=-1)


def mmdit_block(x_img, x_txt, temb, w, heads, eps=1e-6, return_parts=False, txt_pre_only=False):
    """One joint image+text block.

    x_img[B, Ni, D], x_txt[B, Nt, D], temb[B, D]; w = {'img': {...}, 'txt': {...}} with
    ada_w/b [6D, D], qkv_w/b [3D, D], out_w/b [D, D], fc1_w/b [4D, D], fc2_w/b [D, 4D].
    Both streams are modulated, projected to q/k/v with their own weights, attend
    jointly over the concatenated (image first) token sequence, and then each stream
    applies its own output projection and MLP with gated residuals.  With txt_pre_only (the last
    block of a model, whose text output nothing reads) the text stream only takes part in the
    attention and is returned unchanged."""
    xs = {'img': _f64(x_img), 'txt': _f64(x_txt)}
    temb = _f64(temb)
    mods, qkv = {}, {}
    for s in ('img', 'txt'):
        mods[s] = adaln_modulation(temb, w[s]['ada_w'], w[s]['ada_b'], 6)
        sh1, sc1 = mods[s][0], mods[s][1]
        h = modulate(layer_norm(xs[s], eps), sh1, sc1)
        y = linear(h, w[s]['qkv_w'], w[s]['qkv_b'])
        qkv[s] = [split_heads(part, heads) for part in np.split(y, 3, axis=-1)]
    q, k, v = (np.concatenate([qkv['img'][i], qkv['txt'][i]], axis=2) for i in range(3))
    o = attention(q, k, v)
    Ni = xs['img'].shape[1]
    os_ = {'img': o[:, :Ni], 'txt': o[:, Ni:]}
    out = {}
    for s in ('img', 'txt'):
        if s == 'txt' and txt_pre_only:
            out[s] = xs[s]
            continue
        _, _, g1, sh2, sc2, g2 = mods[s]
        x = xs[s] + g1[:, None, :] * linear(os_[s], w[s]['out_w'], w[s]['out_b'])
        h2 = modulate(layer_norm(x, eps), sh2, sc2)
        m = linear(gelu_tanh(linear(h2, w[s]['fc1_w'], w[s]['fc1_b'])), w[s]['fc2_w'], w[s]['fc2_b'])
        out[s] = x + g2[:, None, :] * m
    if return_parts:
        return out['img'], out['txt'], {'q': q, 'k': k, 'v': v, 'o': o}
    return out['img'], out['txt']


def mmdit_block_rows(x_img, x_txt, temb, w, heads, img_rows, txt_rows, eps=1e-6):
    """The same block, evaluated only for the listed token rows of each stream (sampled outputs at
    sizes where the full block is too slow): keys and values are formed for ALL tokens, queries,
    attention, projections and MLP only for the selected rows (everything after the attention is
    per token).  Returns (out_img[B, len(img_rows), D], out_txt[B, len(txt_rows), D])."""
    xs = {'img': _f64(x_img), 'txt': _f64(x_txt)}
    rows = {'img': np.asarray(img_rows, dtype=np.int64), 'txt': np.asarray(txt_rows, dtype=np.int64)}
    temb = _f64(temb)
    mods, ks, vs, qs = {}, [], [], []
    for s in ('img', 'txt'):
        mods[s] = adaln_modulation(temb, w[s]['ada_w'], w[s]['ada_b'], 6)
        h = modulate(layer_norm(xs[s], eps), mods[s][0], mods[s][1])
        y = linear(h, w[s]['qkv_w'], w[s]['qkv_b'])
        q, k, v = (split_heads(part, heads) for part in np.split(y, 3, axis=-1))
        qs.append(q[:, :, rows[s]])
        ks.append(k)
        vs.append(v)
    o = attention(np.concatenate(qs, axis=2), np.concatenate(ks, axis=2), np.concatenate(vs, axis=2))
    n_sel = len(rows['img'])
    os_ = {'img': o[:, :n_sel], 'txt': o[:, n_sel:]}
    out = {}
    for s in ('img', 'txt'):
        _, _, g1, sh2, sc2, g2 = mods[s]
        x = xs[s][:, rows[s]] + g1[:, None, :] * linear(os_[s], w[s]['out_w'], w[s]['out_b'])
        h2 = modulate(layer_norm(x, eps), sh2, sc2)
        m = linear(gelu_tanh(linear(h2, w[s]['fc1_w'], w[s]['fc1_b'])), w[s]['fc2_w'], w[s]['fc2_b'])
        out[s] = x + g2[:, None, :] * m
    return out['img'], out['txt']


def mmdit_embed(latent, ctx, t, P, patch, pooled=None):
    """Token / context / timestep embeddings of the branch forward.  With a pooled text vector
    pooled[B, pooled_dim], its projection W_p2 SiLU(W_p1 pooled + b_p1) + b_p2 is added to the
    timestep embedding, so that the modulation of every block also depends on the prompt."""
    x_img = linear(patchify(latent, patch), P['pe_w'], P['pe_b']) + _f64(P['pos'])[None]
    x_txt = linear(ctx, P['ce_w'], P['ce_b'])
    temb = timestep_mlp(t, P['t1_w'], P['t1_b'], P['t2_w'], P['t2_b'], P['t1_w'].shape[1])
    if pooled is not None:
        temb = temb + linear(silu(linear(pooled, P['p1_w'], P['p1_b'])), P['p2_w'], P['p2_b'])
    return x_img, x_txt, temb


def mmdit_final(x_img, temb, P, Hh, Ww, C, patch, eps=1e-6):
    """Final adaLN (shift, scale) LayerNorm, linear to patch pixels, unpatchify."""
    sh, sc = adaln_modulation(temb, P['f_ada_w'], P['f_ada_b'], 2)
    y = modulate(layer_norm(x_img, eps), sh, sc)
    return unpatchify(linear(y, P['f_w'], P['f_b']), Hh, Ww, C, patch)


def mmdit_forward(latent, ctx, t, P, blocks, heads, patch, txt_pre_only_last=False, pooled=None):
    """One guidance-branch denoiser evaluation v = f_theta(x_t, c, t) (Sec. 4.1).

    latent[B, Hh, Ww, C], ctx[B, Nt, ctx_dim], t[B]; `blocks` is an iterable of per-block
    weight dicts (may be a generator so that large models are streamed).  txt_pre_only_last runs
    the last block with a text stream that only supplies keys and values; pooled[B, pooled_dim]
    is the optional pooled text vector (see mmdit_embed)."""
    B, Hh, Ww, C = np.shape(latent)
    x_img, x_txt, temb = mmdit_embed(latent, ctx, t, P, patch, pooled)
    it = iter(blocks)
    w = next(it, None)
    while w is not None:
        nxt = next(it, None)
        x_img, x_txt = mmdit_block(x_img, x_txt, temb, w, heads, txt_pre_only=txt_pre_only_last and nxt is None)
        w = nxt
    return mmdit_final(x_img, temb, P, Hh, Ww, C, patch)


# --------------------------------------------------------------------------------------
# SDXL-shaped transformer stage block (layout: a reading of the workload text; parity
# unpinned by the paper)
# --------------------------------------------------------------------------------------
def sdxl_block(x, ctx, w, heads):
    """x[B, T, C], ctx[B, Tc, ctx_dim].

    g = GroupNorm32(x); a = g + SelfAttn(LN(g)); b = a + CrossAttn(LN(a), ctx);
    c = b + W2 (u * GELUerf(gate)) + b2 with [u, gate] = split(LN(b) W1^T + b1);
    out = x + c.  q/k/v projections carry no bias, output projections do."""
    x = _f64(x)
    g = group_norm(x, 32, w['gn_g'], w['gn_b'], 1e-5)
    h = layer_norm_affine(g, w['ln1_g'], w['ln1_b'])
    q, k, v = (split_heads(linear(h, w[n]), heads) for n in ('q1_w', 'k1_w', 'v1_w'))
    a = g + linear(attention(q, k, v), w['o1_w'], w['o1_b'])
    h = layer_norm_affine(a, w['ln2_g'], w['ln2_b'])
    q = split_heads(linear(h, w['q2_w']), heads)
    k = split_heads(linear(ctx, w['k2_w']), heads)
    v = split_heads(linear(ctx, w['v2_w']), heads)
    b = a + linear(attention(q, k, v), w['o2_w'], w['o2_b'])
    h = layer_norm_affine(b, w['ln3_g'], w['ln3_b'])
    u, gate = np.split(linear(h, w['ff1_w'], w['ff1_b']), 2, axis=-1)
    c = b + linear(u * gelu_erf(gate), w['ff2_w'], w['ff2_b'])
    return x + c


def sdxl_block_rows(x, ctx, w, heads, rows):
    """The same block for the listed token rows only (sampled outputs at sizes where the full block is
    too slow): the group statistics, and the self-attention keys and values, are formed from ALL tokens;
    queries and everything after the self-attention only for the selected rows (cross-attention keys come
    from the context, the rest is per token).  Returns out[B, len(rows), C]."""
    x = _f64(x)
    rows = np.asarray(rows, dtype=np.int64)
    g = group_norm(x, 32, w['gn_g'], w['gn_b'], 1e-5)
    h = layer_norm_affine(g, w['ln1_g'], w['ln1_b'])
    k = split_heads(linear(h, w['k1_w']), heads)
    v = split_heads(linear(h, w['v1_w']), heads)
    q = split_heads(linear(h[:, rows], w['q1_w']), heads)
    a = g[:, rows] + linear(attention(q, k, v), w['o1_w'], w['o1_b'])
    h = layer_norm_affine(a, w['ln2_g'], w['ln2_b'])
    q = split_heads(linear(h, w['q2_w']), heads)
    k = split_heads(linear(ctx, w['k2_w']), heads)
    v = split_heads(linear(ctx, w['v2_w']), heads)
    b = a + linear(attention(q, k, v), w['o2_w'], w['o2_b'])
    h = layer_norm_affine(b, w['ln3_g'], w['ln3_b'])
    u, gate = np.split(linear(h, w['ff1_w'], w['ff1_b']), 2, axis=-1)
    c = b + linear(u * gelu_erf(gate), w['ff2_w'], w['ff2_b'])
    return x[:, rows] + c


# --------------------------------------------------------------------------------------
# Guidance, discrepancy, scheduler (the parts the paper states explicitly)
# --------------------------------------------------------------------------------------
def cfg_combine(v_c, v_u, s):
    """Classifier-free guidance (Sec. 3, CFG equation): eps_cfg = eps_c + w (eps_c - eps_u).
    Parameterised by s = 1 + w, i.e. v = v_u + s (v_c - v_u): s = 1 gives the conditional
    prediction, s = 0 the unconditional one."""
    v_c, v_u = _f64(v_c), _f64(v_u)
    return v_u + s * (v_c - v_u)


def cfg_combine_w(v_c, v_u, w):
    """The paper's own parameterisation with guidance weight w."""
    v_c, v_u = _f64(v_c), _f64(v_u)
    return v_c + w * (v_c - v_u)


def branch_discrepancy(v_c, v_u, p=1):
    """Denoising discrepancy per sample (Eq. 1; Alg. 1 step computing M_t; velocity form of
    Sec. 4.2 for flow matching): ||v_c - v_u||_p / ||v_u||_p over all elements of a sample.
    p = 1 is the paper's rel-MAE, p = 2 the rel-L2 variant of the workload configs.
    v_c, v_u: [B, ...] -> [B].  0/0 -> 0, x/0 -> +inf for x > 0."""
    v_c, v_u = _f64(v_c), _f64(v_u)
    B = v_c.shape[0]
    d = (v_c - v_u).reshape(B, -1)
    u = v_u.reshape(B, -1)
    if p == 1:
        num, den = np.abs(d).sum(axis=1), np.abs(u).sum(axis=1)
    elif p == 2:
        num, den = np.sqrt((d * d).sum(axis=1)), np.sqrt((u * u).sum(axis=1))
    else:
        raise ValueError("p must be 1 or 2")
    out = np.empty(B, dtype=F64)
    for b in range(B):
        if num[b] == 0.0:
            out[b] = 0.0
        elif den[b] == 0.0:
            out[b] = np.inf
        else:
            out[b] = num[b] / den[b]
    return out


def euler_step(x, v, t, t_next):
    """Explicit Euler step of dx/dt = v (Sec. 3, flow matching): x + (t_next - t) v."""
    return _f64(x) + (float(t_next) - float(t)) * _f64(v)


def affine_step(x, e, a, b):
    """Generic affine scheduler update a x + b e (covers Euler (1, dt), DDIM and the
    CFG-adjusted reverse mean of Sec. 3, all affine in (x, eps))."""
    return float(a) * _f64(x) + float(b) * _f64(e)


def sigma_schedule(T, shift):
    """Shifted linear flow-matching schedule: u_i = 1 - i/T, sigma_i = a u_i / (1 + (a-1) u_i),
    i = 0..T (sigma_0 = 1, sigma_T = 0); integrates from t = 1 to t = 0 (Sec. 3)."""
    u = 1.0 - np.arange(T + 1, dtype=F64) / T
    return shift * u / (1.0 + (shift - 1.0) * u)


def guided_step(x, v_c, v_u, s, t, t_next):
    """CFG combine, both discrepancies and the Euler update for one denoising step.
    x, v_c, v_u: [B, ...].  Returns (x_next, v, disc_l1[B], disc_l2[B])."""
    v = cfg_combine(v_c, v_u, s)
    return euler_step(x, v, t, t_next), v, branch_discrepancy(v_c, v_u, 1), branch_discrepancy(v_c, v_u, 2)


def sampling_loop(latent, ctx_c, ctx_u, P, blocks_fn, heads, patch, T, shift, s):
    """Guided flow-matching sampling (Alg. 1 without the stage switch): each step evaluates
    both branches, records the discrepancies, combines and steps.  blocks_fn() returns a
    fresh iterable of block weights.  Returns (x_0, M_l1[T], M_l2[T])."""
    x = _f64(latent)
    sig = sigma_schedule(T, shift)
    M1, M2 = [], []
    for i in range(T):
        t = np.full(x.shape[0], sig[i])
        v_c = mmdit_forward(x, ctx_c, t, P, blocks_fn(), heads, patch)
        v_u = mmdit_forward(x, ctx_u, t, P, blocks_fn(), heads, patch)
        x, _, d1, d2 = guided_step(x, v_c, v_u, s, sig[i], sig[i + 1])
        M1.append(d1)
        M2.append(d2)
    return x, np.array(M1), np.array(M2)


# --------------------------------------------------------------------------------------
# Adaptive switching rule (Sec. 4.3, Eq. 2-3, Alg. 1), in ascending step index i = 0..T-1
# --------------------------------------------------------------------------------------
def switching_points(M, L, g_slope, tau_cap, k):
    """Given the discrepancy history M[0..T-1] in sampling order (T = len(M)), return (tau1, tau2).

    The slope over the last L steps is taken as the rate of decline G_i = (M[i-L] - M[i]) / L
    (Eq. 2 read on an ascending step index so that a falling curve gives G >= 0).  tau1' is the
    first i >= L with 0 <= G_i < g_slope; tau1 = min(tau1', cap), and tau1 = cap when the test
    never fires (safety cap); tau2 = tau1 + k (Eq. 3).

    Eq. 3 bounds the interval by 1 <= k < T - tau1, i.e. tau2 must be a step of the run
    (tau2 <= T - 1) so that a fully-connecting stage exists.  The safety cap is an upper bound of
    tau1 (Sec. 4.3), so the cap in force is cap = min(tau_cap, T - 1 - k): with it Eq. 3 holds for
    every history, also for runs shorter than tau_cap + k + 1 steps (the 28-step schedule under
    the printed SD3 setting tau_cap = 40).  k >= T leaves no admissible tau1: ValueError."""
    M = _f64(M)
    T = len(M)
    if k < 1 or k > T - 1:
        raise ValueError("Eq. 3 needs 1 <= k < T - tau1 for some tau1 >= 0: k = %d, T = %d" % (k, T))
    cap = min(tau_cap, T - 1 - k)
    tau1 = None
    for i in range(L, T):
        G = (M[i - L] - M[i]) / L
        if 0.0 <= G < g_slope:
            tau1 = min(i, cap)
            break
    if tau1 is None:
        tau1 = cap
    return tau1, tau1 + k


def stage_of(i, tau1, tau2):
    """Stage of step i: 0 warm-up (i <= tau1), 1 parallelism (tau1 < i < tau2),
    2 fully-connecting (i >= tau2) (Sec. 4.2)."""
    if i <= tau1:
        return 0
    if i < tau2:
        return 1
    return 2
