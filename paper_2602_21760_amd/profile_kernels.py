"""Driver for hardware-counter runs: launches a calibration copy, the fused guidance pass, attention, the GEMM
shapes and one joint block of the SD3-shaped 1024x1024 workload through the C entry points (see profiles/)."""
import sys, os
sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))  # repo root
import torch
from paper_2602_21760_amd import binding as hb

hb.lib()
# calibration: plain copy of 1 GiB (reads 1 GiB, writes 1 GiB)
a = torch.empty(1 << 28, device="cuda", dtype=torch.float32).normal_()
b = torch.empty_like(a)
for _ in range(3):
    b.copy_(a)
torch.cuda.synchronize()
del a, b
# fused guidance pass at the roofline shape
batch, n = 256, 262144
v_c = torch.randn(batch, n, device="cuda").to(torch.bfloat16)
v_u = torch.randn(batch, n, device="cuda").to(torch.bfloat16)
x = torch.randn(batch, n, device="cuda")
xo = torch.empty_like(x)
d1, d2 = torch.empty(batch, device="cuda"), torch.empty(batch, device="cuda")
ws = torch.empty(hb.hyb_discrepancy_workspace_bytes(batch, n), device="cuda", dtype=torch.uint8)
for _ in range(3):
    hb.hyb_cfg_disc_euler(v_c, v_u, x, xo, 7.0, 0.5, 0.45, d1, d2, ws)
torch.cuda.synchronize()
del v_c, v_u, x, xo
# attention and the four GEMMs at the cfg-2 shapes
B, H, N = 1, 24, 4429
q, k, v = (torch.randn(B, H, N, 64, device="cuda").to(torch.bfloat16) for _ in range(3))
o = torch.empty(B, N, H * 64, device="cuda", dtype=torch.bfloat16)
for _ in range(3):
    hb.hyb_joint_attention(q, k, v, o)
M = 4429
for n_, k_, epi in ((4608, 1536, hb.HYB_EPI_BIAS), (6144, 1536, hb.HYB_EPI_GELU_TANH), (1536, 6144, hb.HYB_EPI_GATE_RESIDUAL)):
    a = torch.randn(M, k_, device="cuda").to(torch.bfloat16)
    w = (torch.randn(n_, k_, device="cuda") * 0.02).to(torch.bfloat16)
    bias = torch.randn(n_, device="cuda")
    res = torch.randn(M, n_, device="cuda")
    out = torch.empty(M, n_, device="cuda", dtype=torch.float32 if epi == hb.HYB_EPI_GATE_RESIDUAL else torch.bfloat16)
    kw = dict(residual=res) if epi == hb.HYB_EPI_GATE_RESIDUAL else {}
    for _ in range(3):
        hb.hyb_linear(a, w, bias, out, epi, **kw)
torch.cuda.synchronize()
# one joint block of the same workload through hyb_block_forward: there the attention kernel may split its last
# query blocks along the keys (it has the block's workspace for the partial results) and a merge kernel follows
from paper_2602_21760_amd import synth
cfg = synth.CFG2
D = cfg.hidden
wnp = synth.mmdit_block_weights(cfg, 0)
devw = {s: {n_: torch.from_numpy(a_).cuda().to(torch.bfloat16 if n_.endswith("_w") else torch.float32) for n_, a_ in wnp[s].items()
            if not n_.startswith("ada_")} for s in wnp}
desc = hb.block_desc(1, cfg.n_img, cfg.n_txt, D, cfg.heads, hb.HYB_BF16)
ws = torch.empty(max(hb.hyb_block_workspace_bytes(desc), 256), device="cuda", dtype=torch.uint8)
xi, xt = torch.randn(1, cfg.n_img, D, device="cuda"), torch.randn(1, cfg.n_txt, D, device="cuda")
mod = torch.randn(1, 12 * D, device="cuda") * 0.1
for _ in range(3):
    hb.hyb_block_forward(desc, hb.block_weights(devw["img"], devw["txt"]), xi, xt, mod, mod[:, 6 * D:], 12 * D, xi, xt, ws)
torch.cuda.synchronize()
print("done")
