"""GPU parity at the full workload sizes, in the launch configuration the benchmark times: whole-
output comparison where the oracle finishes in about two minutes (the SD3-shaped 1024x1024 branch
forward), sampled outputs elsewhere (attention rows at 4429 and 16717 tokens, GEMM rows at the real
shapes), and one guided step at full token count with a reduced block count."""
import time

import numpy as np
import pytest
import torch

from oracle import hyb_oracle as O
from paper_2602_21760_amd import synth
from gpu_util import TOL_BF16, TOL_DISC, dev, err, host, rel_l2, worst_row

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hb():
    from paper_2602_21760_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("shape", [(2, 24, 4429), (1, 24, 16717), (1, 24, 25933)])
def test_attention_full_size_sampled_rows(hb, shape):
    B, H, N = shape
    q, k, v = (synth.normal(60 + i, (B, H, N, 64), 1.0, "bf16") for i in range(3))
    o = torch.empty(B, N, H * 64, device="cuda", dtype=torch.bfloat16)
    hb.hyb_joint_attention(dev(q, torch.bfloat16), dev(k, torch.bfloat16), dev(v, torch.bfloat16), o)
    rows = np.unique(np.concatenate([[0, 1, 31, 32, 127, 128, N - 334, N - 333, N - 2, N - 1],
                                     np.random.default_rng(0).integers(0, N, 40)]))
    ref = O.attention(q, k, v, rows=rows)
    assert err(host(o)[:, rows], ref) < 1e-2


# the four GEMMs of a joint block at the batch-2 row counts (image rows; text rows ride in the same launch)
@pytest.mark.parametrize("nk", [(4608, 1536), (1536, 1536), (6144, 1536), (1536, 6144)])
def test_linear_full_shapes_sampled_rows(hb, nk):
    n, k = nk
    m = 8192 + 77
    a, w, b = synth.normal(70, (m, k), 1.0, "bf16"), synth.normal(71, (n, k), 0.02, "bf16"), synth.normal(72, (n,), 0.02, "f32")
    out = torch.empty(m, n, device="cuda", dtype=torch.bfloat16)
    hb.hyb_linear(dev(a, torch.bfloat16), dev(w, torch.bfloat16), dev(b), out, hb.HYB_EPI_GELU_TANH)
    rows = np.unique(np.concatenate([[0, 127, 128, 255, 256, m - 78, m - 77, m - 1], np.random.default_rng(1).integers(0, m, 48)]))
    ref = O.gelu_tanh(O.linear(a[rows], w, b))
    assert err(host(out)[rows], ref) < 1e-2


@pytest.mark.timeout(600)
def test_guided_step_full_tokens_reduced_depth(hb):
    """Batch 2 (cond + uncond) at 4096 + 333 tokens and hidden 1536, 2 blocks, then the fused pass."""
    from paper_2602_21760_amd import model
    cfg = synth.scaled(synth.CFG3, blocks=2)
    P = synth.mmdit_globals(cfg)
    blocks = list(synth.mmdit_blocks(cfg))
    lat, ctx_c, ctx_u = synth.mmdit_inputs(cfg)
    m = model.MMDiT(cfg, P, blocks)
    gs = model.GuidedSampler(m, cfg.guidance)
    sig = O.sigma_schedule(cfg.steps, cfg.shift)
    x = dev(lat).clone()
    gs.step(x, dev(np.stack([ctx_c, ctx_u])), float(sig[0]), float(sig[1]), 0)
    v_gpu = host(m.v)
    tt = np.full(2, np.float32(sig[0]))
    ref_v = O.mmdit_forward(np.stack([lat, lat]), np.stack([ctx_c, ctx_u]), tt, P, blocks, cfg.heads, cfg.patch)
    assert err(v_gpu, ref_v) < TOL_BF16
    rx, _, r1, r2 = O.guided_step(lat[None], ref_v[0:1], ref_v[1:2], cfg.guidance, np.float32(sig[0]), np.float32(sig[1]))
    assert err(host(x), rx[0]) < TOL_BF16
    # discrepancy on IDENTICAL branch outputs (the GPU's bf16 velocities fed to both reductions)
    t1, t2 = O.branch_discrepancy(v_gpu[0:1], v_gpu[1:2], 1)[0], O.branch_discrepancy(v_gpu[0:1], v_gpu[1:2], 2)[0]
    g1, g2 = gs.disc[0, 0].item(), gs.disc[1, 0].item()
    assert abs(g1 - t1) < TOL_DISC * t1 and abs(g2 - t2) < TOL_DISC * t2
    print("end-to-end discrepancy gpu (L1, L2) = (%.5f, %.5f), oracle = (%.5f, %.5f)" % (g1, g2, r1[0], r2[0]))


@pytest.mark.timeout(1500)
def test_cfg2_full_forward(hb, capsys):
    """One full denoiser forward of the SD3-shaped branch (24 blocks) against the fp64 oracle.
    The oracle needs minutes of CPU time here, so progress lines go to the real stdout."""
    from paper_2602_21760_amd import model
    cfg = synth.CFG2
    P = synth.mmdit_globals(cfg)
    lat, ctx_c, _ = synth.mmdit_inputs(cfg)
    tt = np.full(1, 0.5, dtype=np.float32)
    t0 = time.time()
    blocks = []
    for i in range(cfg.blocks):
        blocks.append(synth.mmdit_block_weights(cfg, i))
        if i % 8 == 7:
            with capsys.disabled():
                print("  [cfg2 full] generated weights of %d blocks, %.0f s" % (i + 1, time.time() - t0), flush=True)
    m = model.MMDiT(cfg, P, blocks)
    v = host(m.forward(dev(lat[None]), dev(ctx_c[None]), dev(tt)))
    del m
    torch.cuda.empty_cache()
    # the oracle's branch forward, written out block by block only to report progress
    x_img, x_txt, temb = O.mmdit_embed(lat[None], ctx_c[None], tt, P, cfg.patch)
    for i, w in enumerate(blocks):
        x_img, x_txt = O.mmdit_block(x_img, x_txt, temb, w, cfg.heads)
        if i % 4 == 3:
            with capsys.disabled():
                print("  [cfg2 full] oracle block %d / %d, %.0f s" % (i + 1, cfg.blocks, time.time() - t0), flush=True)
    ref = O.mmdit_final(x_img, temb, P, cfg.latent_hw, cfg.latent_hw, cfg.latent_c, cfg.patch)
    e_all, e_row = rel_l2(v, ref), worst_row(v, ref)
    with capsys.disabled():
        print("  [cfg2 full] v vs oracle: rel-L2 %.3e, worst latent line %.3e (%.0f s)" % (e_all, e_row, time.time() - t0), flush=True)
    assert err(v, ref) < TOL_BF16


@pytest.mark.timeout(900)
@pytest.mark.parametrize("cfg", [synth.CFG4, synth.CFG6], ids=["cfg4_2048", "cfg6_2560"])
def test_block_high_resolution_sampled_rows(hb, capsys, cfg):
    """One joint block at the 2048 x 2048 and 2560 x 2560 shapes (16384 / 25600 image + 333 text tokens,
    hidden 1536): the GPU block output is compared on sampled token rows that the oracle evaluates one by
    one (keys / values of all tokens, queries and everything after the attention for the sampled rows only)."""
    from paper_2602_21760_amd import binding as B
    D = cfg.hidden
    w = synth.mmdit_block_weights(cfg, 0)
    x_img = synth.normal(91, (1, cfg.n_img, D), 1.0, "f32")
    x_txt = synth.normal(92, (1, cfg.n_txt, D), 1.0, "f32")
    temb = synth.normal(93, (1, D), 1.0, "f32")
    devw = {s: {n: dev(a, torch.bfloat16 if n.endswith("_w") else torch.float32) for n, a in w[s].items()} for s in w}
    mod = torch.empty(1, 12 * D, device="cuda")
    hb.hyb_adaln_modulation(torch.cat([devw["img"]["ada_w"], devw["txt"]["ada_w"]]).contiguous(),
                            torch.cat([devw["img"]["ada_b"], devw["txt"]["ada_b"]]).contiguous(), dev(temb), mod)
    desc = B.block_desc(1, cfg.n_img, cfg.n_txt, D, cfg.heads, B.HYB_BF16)
    ws = torch.empty(hb.hyb_block_workspace_bytes(desc), device="cuda", dtype=torch.uint8)
    xi, xt = dev(x_img), dev(x_txt)
    hb.hyb_block_forward(desc, B.block_weights(devw["img"], devw["txt"]), xi, xt, mod, mod[:, 6 * D:], 12 * D, xi, xt, ws)
    g_img, g_txt = host(xi), host(xt)
    rng = np.random.default_rng(4)
    ri = np.unique(np.concatenate([[0, 127, 128, cfg.n_img - 1], rng.integers(0, cfg.n_img, 56)]))
    rt = np.unique(np.concatenate([[0, 255, 256, cfg.n_txt - 1], rng.integers(0, cfg.n_txt, 12)]))
    with capsys.disabled():
        print("  [%s block] GPU done, oracle on %d + %d sampled rows ..." % (cfg.name, len(ri), len(rt)), flush=True)
    r_img, r_txt = O.mmdit_block_rows(x_img, x_txt, temb, w, cfg.heads, ri, rt)
    assert err(g_img[:, ri], r_img) < TOL_BF16 and err(g_txt[:, rt], r_txt) < TOL_BF16
    assert err(g_img[:, ri] - x_img[:, ri], r_img - x_img[:, ri]) < 5e-2
