"""Seeded synthetic inputs and random-init weights for the five workload configurations.

Pure numpy data generation: no arithmetic of the method lives here, so both the CPU oracle
tests and the HIP path may draw their inputs from this module.  Every tensor is float32;
for bf16 workloads the values are rounded to the nearest bf16 (ties to even) once, here,
so that both sides see identical data.

Recipe: weights and biases N(0, 0.02^2) with seed 1000 + tensor index (norm gains are
1 + N(0, 0.02^2)); latent N(0, 1) seed 1; conditional text N(0, 1) seed 2; unconditional
text N(0, 1) seed 3; positional table N(0, 0.02^2) seed 4.
"""
from dataclasses import dataclass

import numpy as np


def round_bf16(a):
    """Round float32 values to the nearest bf16-representable float32 (ties to even)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + r) & np.uint32(0xFFFF0000)).view(np.float32)


@dataclass(frozen=True)
class MMDiTConfig:
    name: str
    blocks: int
    hidden: int
    heads: int
    latent_hw: int
    latent_c: int
    n_txt: int
    ctx_dim: int
    batch: int
    dtype: str            # "f32" or "bf16"
    patch: int = 2
    head_dim: int = 64
    mlp_ratio: int = 4
    temb_dim: int = 256
    steps: int = 1
    shift: float = 3.0
    guidance: float = 7.0
    pooled_dim: int = 0   # > 0: a pooled text vector of this width also conditions the modulation

    @property
    def n_img(self):
        return (self.latent_hw // self.patch) ** 2

    @property
    def patch_dim(self):
        return self.patch * self.patch * self.latent_c

    @property
    def latent_elems(self):
        return self.latent_hw * self.latent_hw * self.latent_c

    def flops_per_sample(self):
        """Algorithmic flops of one branch forward (GEMMs + full NxN attention + adaLN)."""
        D, N = self.hidden, self.n_img + self.n_txt
        per_block = 24 * D * D * N + 4 * N * N * D + 2 * 2 * 6 * D * D
        embed = 2 * self.n_img * self.patch_dim * D * 2 + 2 * self.n_txt * self.ctx_dim * D
        return self.blocks * per_block + embed


@dataclass(frozen=True)
class SDXLStageConfig:
    name: str
    blocks: int
    tokens: int
    channels: int
    heads: int
    n_ctx: int = 77
    ctx_dim: int = 2048
    batch: int = 2
    dtype: str = "bf16"

    def flops_per_sample(self):
        C, T, S = self.channels, self.tokens, self.n_ctx
        per_block = 2 * T * C * C * 4 + 4 * T * T * C            # self attention
        per_block += 2 * T * C * C * 2 + 2 * 2 * S * self.ctx_dim * C + 4 * T * S * C   # cross
        per_block += 2 * T * C * 8 * C + 2 * T * 4 * C * C       # GEGLU feed-forward
        return self.blocks * per_block


CFG1 = MMDiTConfig("cfg1_tiny_f32", blocks=1, hidden=256, heads=4, latent_hw=16, latent_c=4,
                   n_txt=16, ctx_dim=256, batch=2, dtype="f32")
CFG2 = MMDiTConfig("cfg2_sd3_1024_bf16", blocks=24, hidden=1536, heads=24, latent_hw=128,
                   latent_c=16, n_txt=333, ctx_dim=4096, batch=1, dtype="bf16")
CFG3 = MMDiTConfig("cfg3_sd3_guided_loop_bf16", blocks=24, hidden=1536, heads=24, latent_hw=128,
                   latent_c=16, n_txt=333, ctx_dim=4096, batch=2, dtype="bf16", steps=28)
CFG4 = MMDiTConfig("cfg4_sd3_2048_bf16", blocks=24, hidden=1536, heads=24, latent_hw=256,
                   latent_c=16, n_txt=333, ctx_dim=4096, batch=1, dtype="bf16")
# the largest resolution of the paper's high-resolution study (Appendix, SD3 at 2560 x 2560): 25600 image tokens
CFG6 = MMDiTConfig("cfg6_sd3_2560_bf16", blocks=24, hidden=1536, heads=24, latent_hw=320,
                   latent_c=16, n_txt=333, ctx_dim=4096, batch=1, dtype="bf16")
CFG5A = SDXLStageConfig("cfg5_sdxl_stageA", blocks=10, tokens=4096, channels=640, heads=10)
CFG5B = SDXLStageConfig("cfg5_sdxl_stageB", blocks=20, tokens=1024, channels=1280, heads=20)
# the same two stages at 2048 x 2048 (4 x the tokens)
CFG7A = SDXLStageConfig("sdxl_2048_stageA", blocks=10, tokens=16384, channels=640, heads=10)
CFG7B = SDXLStageConfig("sdxl_2048_stageB", blocks=20, tokens=4096, channels=1280, heads=20)
CFG5_LATENT = (128, 128, 4)
CFG5_GUIDANCE = 5.0


def scaled(cfg, **kw):
    """A copy of a config with some fields replaced (reduced-size parity cases)."""
    d = dict(cfg.__dict__)
    d.update(kw)
    return type(cfg)(**d)


def _finish(a, dtype):
    a = a.astype(np.float32)
    return round_bf16(a) if dtype == "bf16" else a


def normal(seed, shape, std=1.0, dtype="f32", mean=0.0):
    rng = np.random.default_rng(seed)
    a = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    if mean != 0.0:
        a += np.float32(mean)
    return _finish(a, dtype)


_STREAM_TENSORS = (("ada_w", 6, 1), ("ada_b", 6, 0), ("qkv_w", 3, 1), ("qkv_b", 3, 0),
                   ("out_w", 1, 1), ("out_b", 1, 0), ("fc1_w", 4, 1), ("fc1_b", 4, 0),
                   ("fc2_w", 1, 4), ("fc2_b", 1, 0))


def mmdit_globals(cfg):
    """Embedding / final-layer weights (tensor indices 0..11)."""
    D, dt = cfg.hidden, cfg.dtype
    shapes = [("pe_w", (D, cfg.patch_dim)), ("pe_b", (D,)), ("ce_w", (D, cfg.ctx_dim)), ("ce_b", (D,)),
              ("t1_w", (D, cfg.temb_dim)), ("t1_b", (D,)), ("t2_w", (D, D)), ("t2_b", (D,)),
              ("f_ada_w", (2 * D, D)), ("f_ada_b", (2 * D,)), ("f_w", (cfg.patch_dim, D)),
              ("f_b", (cfg.patch_dim,))]
    if cfg.pooled_dim:   # tensor indices 12..15
        shapes += [("p1_w", (D, cfg.pooled_dim)), ("p1_b", (D,)), ("p2_w", (D, D)), ("p2_b", (D,))]
    P = {n: normal(1000 + i, s, 0.02, dt) for i, (n, s) in enumerate(shapes)}
    P["pos"] = normal(4, (cfg.n_img, D), 0.02, dt)
    return P


def mmdit_block_weights(cfg, i):
    """Weights of joint block i: {'img': {...}, 'txt': {...}} (tensor indices from 100 + 20 i)."""
    D, dt = cfg.hidden, cfg.dtype
    w = {}
    for si, s in enumerate(("img", "txt")):
        d = {}
        for ti, (n, om, im) in enumerate(_STREAM_TENSORS):
            out_f = om * D
            shape = (out_f, im * D) if im else (out_f,)
            d[n] = normal(1000 + 100 + 20 * i + 10 * si + ti, shape, 0.02, dt)
        w[s] = d
    return w


def mmdit_blocks(cfg):
    """Generator over the block weights (streams them, a full SD3-shaped set is ~8 GB in f32)."""
    for i in range(cfg.blocks):
        yield mmdit_block_weights(cfg, i)


def mmdit_inputs(cfg):
    """latent[B, Hh, Ww, C] (the same latent for every batch row: both guidance branches start
    from one x_t), ctx_c / ctx_u[Nt, ctx_dim] for the conditional / unconditional text."""
    lat = normal(1, (cfg.latent_hw, cfg.latent_hw, cfg.latent_c), 1.0, cfg.dtype)
    ctx_c = normal(2, (cfg.n_txt, cfg.ctx_dim), 1.0, cfg.dtype)
    ctx_u = normal(3, (cfg.n_txt, cfg.ctx_dim), 1.0, cfg.dtype)
    return lat, ctx_c, ctx_u


def mmdit_pooled(cfg):
    """Pooled text vectors [pooled_dim] of the conditional / unconditional prompt (seeds 5, 6)."""
    return normal(5, (cfg.pooled_dim,), 1.0, cfg.dtype), normal(6, (cfg.pooled_dim,), 1.0, cfg.dtype)


_SDXL_TENSORS = ("gn_g", "gn_b", "ln1_g", "ln1_b", "q1_w", "k1_w", "v1_w", "o1_w", "o1_b",
                 "ln2_g", "ln2_b", "q2_w", "k2_w", "v2_w", "o2_w", "o2_b",
                 "ln3_g", "ln3_b", "ff1_w", "ff1_b", "ff2_w", "ff2_b")


def sdxl_block_weights(cfg, i, base=5000):
    C, X, dt = cfg.channels, cfg.ctx_dim, cfg.dtype
    shapes = {"q1_w": (C, C), "k1_w": (C, C), "v1_w": (C, C), "o1_w": (C, C), "q2_w": (C, C),
              "k2_w": (C, X), "v2_w": (C, X), "o2_w": (C, C), "ff1_w": (8 * C, C), "ff1_b": (8 * C,),
              "ff2_w": (C, 4 * C)}
    w = {}
    for ti, n in enumerate(_SDXL_TENSORS):
        seed = base + 40 * i + ti
        if n.endswith("_g"):
            w[n] = normal(seed, (C,), 0.02, dt, mean=1.0)
        else:
            w[n] = normal(seed, shapes.get(n, (C,)), 0.02, dt)
    return w


def sdxl_inputs(cfg, seed_x=1):
    x = normal(seed_x, (cfg.batch, cfg.tokens, cfg.channels), 1.0, cfg.dtype)
    ctx = np.stack([normal(2, (cfg.n_ctx, cfg.ctx_dim), 1.0, cfg.dtype),
                    normal(3, (cfg.n_ctx, cfg.ctx_dim), 1.0, cfg.dtype)])[:cfg.batch]
    return x, ctx


def guidance_inputs(n, batch=1, v_dtype="bf16", seed=11, delta=0.1):
    """Stand-in branch outputs for the guidance step: v_u ~ N(0,1), v_c = v_u + delta N(0,1),
    latent x ~ N(0,1) (float32 master copy)."""
    v_u = normal(seed, (batch, n), 1.0, "f32")
    v_c = v_u + np.float32(delta) * normal(seed + 1, (batch, n), 1.0, "f32")
    x = normal(seed + 2, (batch, n), 1.0, "f32")
    return _finish(v_c, v_dtype), _finish(v_u, v_dtype), x
