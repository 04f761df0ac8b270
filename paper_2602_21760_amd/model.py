"""Drivers that run the denoiser forward and the guided step purely through libhyb calls.

This is marshalling only: weights are uploaded once (torch tensors = device memory), then every
step of the path is a hyb_* call on torch's current stream.  No arithmetic of the method is done
in Python or by torch operators."""
import numpy as np
import torch

from . import binding as hb

_TORCH_DT = {"f32": torch.float32, "bf16": torch.bfloat16}


def _dev(a, dtype=torch.float32):
    """numpy float32 array -> device tensor (bf16 conversion is exact for bf16-representable data)."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t if dtype == torch.float32 else t.to(dtype)


class MMDiT:
    """Device-resident weights + workspaces of one MMDiT-shaped denoiser (see synth.MMDiTConfig)."""

    def __init__(self, cfg, globals_np, blocks_iter, batch=None, txt_pre_only_last=False):
        self.cfg = cfg
        self.txt_pre_only_last = txt_pre_only_last   # skip the dead text-stream work of the last block
        self.B = cfg.batch if batch is None else batch
        self.act = _TORCH_DT[cfg.dtype]
        self.hdt = hb.HYB_BF16 if cfg.dtype == "bf16" else hb.HYB_F32
        D = cfg.hidden
        P = globals_np
        self.g = {n: _dev(P[n], self.act if n.endswith("_w") else torch.float32) for n in P if n != "pos"}
        self.pos = _dev(P["pos"])
        ada_w, ada_b, self.blocks, self._keep = [], [], [], []
        for w in blocks_iter:
            dev = {}
            for s in ("img", "txt"):
                dev[s] = {n: _dev(a, self.act if n.endswith("_w") else torch.float32) for n, a in w[s].items()
                          if not n.startswith("ada_")}
                ada_w.append(_dev(w[s]["ada_w"], self.act))
                ada_b.append(_dev(w[s]["ada_b"]))
            self._keep.append(dev)
            self.blocks.append(hb.block_weights(dev["img"], dev["txt"]))
        ada_w.append(self.g.pop("f_ada_w"))
        ada_b.append(self.g.pop("f_ada_b"))
        self.ada_w = torch.cat(ada_w, dim=0).contiguous()     # [(blocks * 2 * 6 + 2) * D, D]
        self.ada_b = torch.cat(ada_b, dim=0).contiguous()
        self.mod_rows = self.ada_w.shape[0]
        self._alloc()

    def _alloc(self):
        cfg, B, D = self.cfg, self.B, self.cfg.hidden
        f32 = dict(device="cuda", dtype=torch.float32)
        act = dict(device="cuda", dtype=self.act)
        self.desc = hb.block_desc(B, cfg.n_img, cfg.n_txt, D, cfg.heads, self.hdt, cfg.head_dim, cfg.mlp_ratio, 1e-6)
        # the same block with a text stream that only supplies keys and values (used for the last block when
        # txt_pre_only_last is set: nothing reads the text output of the last block)
        self.desc_pre = hb.block_desc(B, cfg.n_img, cfg.n_txt, D, cfg.heads, self.hdt, cfg.head_dim, cfg.mlp_ratio, 1e-6,
                                      txt_pre_only=True)
        self.ws = torch.empty(max(hb.hyb_block_workspace_bytes(self.desc), 256), device="cuda", dtype=torch.uint8)
        self.t_dev = torch.empty(B, **f32)
        self.t_feat = torch.empty(B, cfg.temb_dim, **act)
        self.t_hid = torch.empty(B, D, **act)
        self.temb = torch.empty(B, D, **f32)
        if cfg.pooled_dim:
            self.pooled_act = torch.empty(B, cfg.pooled_dim, **act)
            self.p_hid = torch.empty(B, D, **act)
        self.mod = torch.empty(B, self.mod_rows, **f32)
        self.tok = torch.empty(B, cfg.n_img, cfg.patch_dim, **act)
        self.ctx_act = torch.empty(B, cfg.n_txt, cfg.ctx_dim, **act)
        self.x_img = torch.empty(B, cfg.n_img, D, **f32)
        self.x_txt = torch.empty(B, cfg.n_txt, D, **f32)
        self.y = torch.empty(B, cfg.n_img, D, **act)
        self.out_tok = torch.empty(B, cfg.n_img, cfg.patch_dim, **act)
        self.v = torch.empty(B, cfg.latent_hw, cfg.latent_hw, cfg.latent_c, **act)

    def reconfigure(self, cfg, batch=None, pos_np=None):
        """Re-allocate the activation buffers for another token count / batch of the SAME network
        (weights are kept; a new positional table is needed when the image token count changes)."""
        assert (cfg.hidden, cfg.heads, cfg.blocks, cfg.dtype) == (self.cfg.hidden, self.cfg.heads, self.cfg.blocks, self.cfg.dtype)
        self.cfg = cfg
        self.B = cfg.batch if batch is None else batch
        if pos_np is not None:
            self.pos = _dev(pos_np)
        assert self.pos.shape[0] == cfg.n_img
        self._alloc()

    def embed(self, latent, ctx, t, pooled=None):
        """latent: f32[B, Hh, Ww, C]; ctx: f32[B, Nt, ctx_dim]; t: f32[B]; pooled: f32[B, pooled_dim] when the
        configuration has a pooled text vector (device tensors)."""
        cfg, g = self.cfg, self.g
        hb.hyb_timestep_embedding(t, self.t_feat)
        hb.hyb_linear(self.t_feat, g["t1_w"], g["t1_b"], self.t_hid, hb.HYB_EPI_SILU)
        hb.hyb_linear(self.t_hid, g["t2_w"], g["t2_b"], self.temb, hb.HYB_EPI_BIAS)
        if cfg.pooled_dim:   # temb += W_p2 SiLU(W_p1 pooled + b_p1) + b_p2 (the sum is the residual epilogue)
            hb.hyb_convert(pooled, self.pooled_act)
            hb.hyb_linear(self.pooled_act, g["p1_w"], g["p1_b"], self.p_hid, hb.HYB_EPI_SILU)
            hb.hyb_linear(self.p_hid, g["p2_w"], g["p2_b"], self.temb, hb.HYB_EPI_GATE_RESIDUAL, residual=self.temb)
        hb.hyb_adaln_modulation(self.ada_w, self.ada_b, self.temb, self.mod)
        hb.hyb_patchify(latent, self.tok, cfg.patch)
        for b in range(self.B):    # the positional table is the "residual" of the patch projection
            hb.hyb_linear(self.tok[b], g["pe_w"], g["pe_b"], self.x_img[b], hb.HYB_EPI_GATE_RESIDUAL, residual=self.pos)
        if cfg.n_txt:
            hb.hyb_convert(ctx, self.ctx_act)
            hb.hyb_linear(self.ctx_act.view(-1, cfg.ctx_dim), g["ce_w"], g["ce_b"], self.x_txt.view(-1, cfg.hidden))

    def run_blocks(self, first=0, last=None):
        D = self.cfg.hidden
        last = len(self.blocks) if last is None else last
        for i in range(first, last):
            mi = self.mod[:, (2 * i) * 6 * D:]
            mt = self.mod[:, (2 * i + 1) * 6 * D:]
            desc = self.desc_pre if (self.txt_pre_only_last and i == len(self.blocks) - 1) else self.desc
            hb.hyb_block_forward(desc, self.blocks[i], self.x_img, self.x_txt, mi, mt, self.mod_rows,
                                 self.x_img, self.x_txt, self.ws)

    def final(self):
        cfg, g, D = self.cfg, self.g, self.cfg.hidden
        fo = len(self.blocks) * 2 * 6 * D
        hb.hyb_layernorm_modulate(self.x_img, self.mod[:, fo:], self.mod[:, fo + D:], self.mod_rows, self.y, 1e-6)
        hb.hyb_linear(self.y.view(-1, D), g["f_w"], g["f_b"], self.out_tok.view(-1, cfg.patch_dim))
        hb.hyb_unpatchify(self.out_tok, self.v, cfg.patch)
        return self.v

    def forward(self, latent, ctx, t, pooled=None):
        """One denoiser evaluation for every batch row; returns v[B, Hh, Ww, C] (activation dtype)."""
        self.embed(latent, ctx, t, pooled)
        self.run_blocks()
        return self.final()


class GuidedSampler:
    """Both guidance branches as batch rows 0 (conditional) and 1 (unconditional) of one forward,
    followed by the fused CFG / discrepancy / Euler pass; the latent master copy stays fp32."""

    def __init__(self, model, scale):
        assert model.B == 2
        self.m, self.scale = model, scale
        cfg = model.cfg
        n = cfg.latent_elems
        self.lat2 = torch.empty(2, cfg.latent_hw, cfg.latent_hw, cfg.latent_c, device="cuda", dtype=torch.float32)
        self.t2 = torch.empty(2, device="cuda", dtype=torch.float32)
        self.ws = torch.empty(max(hb.hyb_discrepancy_workspace_bytes(1, n), 256), device="cuda", dtype=torch.uint8)
        self.disc = torch.zeros(2, 64, device="cuda", dtype=torch.float32)   # [l1 | l2][step]

    def step(self, x, ctx2, t, t_next, i=0):
        """x: f32[Hh, Ww, C] master latent (updated in place); ctx2: f32[2, Nt, ctx_dim]."""
        self.lat2[0].copy_(x)
        self.lat2[1].copy_(x)
        self.t2.fill_(t)
        v = self.m.forward(self.lat2, ctx2, self.t2)
        hb.hyb_cfg_disc_euler(v[0:1], v[1:2], x.view(1, -1), x.view(1, -1), self.scale, t, t_next,
                              disc_l1=self.disc[0, i:i + 1], disc_l2=self.disc[1, i:i + 1], workspace=self.ws)
        return x

    def sample(self, x, ctx2, sigmas, switch=None):
        """All steps of a schedule (sigmas: T + 1 values).  With a switching state (hyb_switch_init), the
        denoising discrepancy of every step (Eq. 1: the L1 ratio) is handed to the controller as soon as
        the step's kernels have finished -- one 4-byte read-back per step, as the online rule of Alg. 1
        needs the value before the next step -- and the stage the controller assigns to each step is
        returned: this single-device build runs every step the same way and only records the decision."""
        steps = len(sigmas) - 1
        if self.disc.shape[1] < steps:
            self.disc = torch.zeros(2, steps, device="cuda", dtype=torch.float32)
        stages = []
        for i in range(steps):
            self.step(x, ctx2, float(sigmas[i]), float(sigmas[i + 1]), i)
            if switch is not None:
                stages.append(hb.hyb_switch_push(switch, float(self.disc[0, i].item())))
        return x, stages


class SDXLStage:
    """Device-resident weights + workspace of one SDXL-shaped transformer stage (see synth.SDXLStageConfig).
    The separate q / k / v (and k / v) projection matrices are concatenated once at load time."""

    def __init__(self, cfg, blocks_iter):
        self.cfg = cfg
        self.act = _TORCH_DT[cfg.dtype]
        self.hdt = hb.HYB_BF16 if cfg.dtype == "bf16" else hb.HYB_F32
        self.blocks, self._keep = [], []
        for w in blocks_iter:
            d = {n: _dev(w[n]) for n in ("gn_g", "gn_b", "ln1_g", "ln1_b", "ln2_g", "ln2_b", "ln3_g", "ln3_b")}
            d["w_qkv1"] = _dev(np.concatenate([w["q1_w"], w["k1_w"], w["v1_w"]]), self.act)
            d["w_kv2"] = _dev(np.concatenate([w["k2_w"], w["v2_w"]]), self.act)
            for dst, src in (("w_o1", "o1_w"), ("w_q2", "q2_w"), ("w_o2", "o2_w"), ("w_ff1", "ff1_w"), ("w_ff2", "ff2_w")):
                d[dst] = _dev(w[src], self.act)
            for dst, src in (("b_o1", "o1_b"), ("b_o2", "o2_b"), ("b_ff1", "ff1_b"), ("b_ff2", "ff2_b")):
                d[dst] = _dev(w[src])
            self._keep.append(d)
            self.blocks.append(hb.sdxl_block_weights(d))
        self.desc = hb.sdxl_block_desc(cfg.batch, cfg.tokens, cfg.channels, cfg.heads, cfg.n_ctx, cfg.ctx_dim, self.hdt)
        self.ws = torch.empty(max(hb.hyb_sdxl_block_workspace_bytes(self.desc), 256), device="cuda", dtype=torch.uint8)
        self.ctx_act = torch.empty(cfg.batch, cfg.n_ctx, cfg.ctx_dim, device="cuda", dtype=self.act)

    def forward(self, x, ctx):
        """x: f32[B, T, C] (updated in place); ctx: f32[B, n_ctx, ctx_dim]."""
        hb.hyb_convert(ctx, self.ctx_act)
        for bw in self.blocks:
            hb.hyb_sdxl_block_forward(self.desc, bw, x, self.ctx_act, x, self.ws)
        return x
