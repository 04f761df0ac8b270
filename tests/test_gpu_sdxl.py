"""GPU parity of the SDXL-shaped transformer stage (GroupNorm, affine LayerNorm, self- and cross-
attention, GEGLU feed-forward) against the CPU oracle: the pieces, a reduced block in fp32 and bf16,
the two real stage shapes with one block each, and the guidance step on the 128 x 128 x 4 latent."""
import numpy as np
import pytest
import torch

from oracle import hyb_oracle as O
from paper_2602_21760_amd import synth
from gpu_util import TOL_BF16, TOL_DISC, TOL_F32, dev, err, host, rel_l2, tdt, tol, worst_row

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hb():
    from paper_2602_21760_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("shape", [(2, 37, 640), (1, 300, 1280), (3, 5, 128), (2, 1, 256), (1, 5003, 128), (2, 4096, 640)])
def test_groupnorm(hb, shape):
    B, T, C = shape
    x = synth.normal(80, shape, 2.0, "f32") + 0.7
    g, b = synth.normal(81, (C,), 0.1, "f32", mean=1.0), synth.normal(82, (C,), 0.1, "f32")
    out = torch.empty(B, T, C, device="cuda")
    ws = torch.empty(hb.hyb_groupnorm_workspace_bytes(B, 32), device="cuda", dtype=torch.uint8)
    dx = dev(x)
    hb.hyb_groupnorm(dx, dev(g), dev(b), out, 32, 1e-5, ws)
    assert err(host(out), O.group_norm(x, 32, g, b, 1e-5)) < 1e-5
    hb.hyb_groupnorm(dx, dev(g), dev(b), dx, 32, 1e-5, ws)          # in place
    assert err(host(dx), O.group_norm(x, 32, g, b, 1e-5)) < 1e-5


@pytest.mark.parametrize("od", ["f32", "bf16"])
def test_layernorm_affine(hb, od):
    x = synth.normal(83, (2, 33, 640), 3.0, "f32") - 1.0
    g, b = synth.normal(84, (640,), 0.1, "f32", mean=1.0), synth.normal(85, (640,), 0.1, "f32")
    out = torch.empty(2, 33, 640, device="cuda", dtype=tdt(od))
    hb.hyb_layernorm_affine(dev(x), dev(g), dev(b), out, 1e-5)
    assert err(host(out), O.layer_norm_affine(x, g, b, 1e-5)) < (4e-3 if od == "bf16" else 1e-5)


def _stage_case(cfg, nblocks, scale_w=1.0):
    from paper_2602_21760_amd import model
    blocks = []
    for i in range(nblocks):
        w = synth.sdxl_block_weights(cfg, i)
        if scale_w != 1.0:
            w = {n: (synth.round_bf16(a * scale_w) if (n.endswith("_w") and cfg.dtype == "bf16") else
                     (a * scale_w if n.endswith("_w") else a)) for n, a in w.items()}
        blocks.append(w)
    x, ctx = synth.sdxl_inputs(cfg)
    st = model.SDXLStage(cfg, blocks)
    dx = dev(x)
    st.forward(dx, dev(ctx))
    ref = x
    for w in blocks:
        ref = O.sdxl_block(ref, ctx, w, cfg.heads)
    return host(dx), ref, x


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_sdxl_block_reduced(hb, dt):
    # ragged token count (several tiles + tail), 5 context tokens short of a tile, weights scaled up so that
    # every sub-layer changes the stream noticeably
    cfg = synth.SDXLStageConfig("t", blocks=2, tokens=333, channels=256, heads=4, n_ctx=77, ctx_dim=128, batch=2, dtype=dt)
    got, ref, x = _stage_case(cfg, 2, scale_w=4.0)
    assert err(got, ref) < tol(dt)
    assert err(got - x, ref - x) < (3e-2 if dt == "bf16" else 1e-3)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("stage", ["A", "B"])
def test_sdxl_stage_real_shapes_one_block(hb, stage):
    cfg = synth.CFG5A if stage == "A" else synth.CFG5B
    got, ref, x = _stage_case(cfg, 1)
    assert err(got, ref) < TOL_BF16
    assert err(got - x, ref - x) < 5e-2


@pytest.mark.timeout(900)
@pytest.mark.parametrize("stage", ["A", "B"])
def test_sdxl_stage_real_shapes_whole_chain(hb, capsys, stage):
    """The whole stage at its real shape: all 10 blocks on 4096 tokens x 640 channels / all 20 blocks on 1024 tokens x
    1280 channels, batch 2, chained in place, every output element against the fp64 oracle's chain."""
    import time
    cfg = synth.CFG5A if stage == "A" else synth.CFG5B
    t0 = time.time()
    got, ref, x = _stage_case(cfg, cfg.blocks)
    with capsys.disabled():
        print("  [sdxl stage %s, %d blocks] rel-L2 %.3e, worst row %.3e (%.0f s)" %
              (stage, cfg.blocks, rel_l2(got, ref), worst_row(got, ref), time.time() - t0), flush=True)
    assert err(got, ref) < TOL_BF16
    assert err(got - x, ref - x) < 5e-2


def test_sdxl_block_is_deterministic_with_split_k(hb):
    """At the stage B shape the context K/V projection and the down-projection split their k range over several
    workgroups per tile; the partial sums are added in a fixed order, so two runs agree bit for bit."""
    from paper_2602_21760_amd import model
    cfg = synth.CFG5B
    w = synth.sdxl_block_weights(cfg, 0)
    x, ctx = synth.sdxl_inputs(cfg)
    st = model.SDXLStage(cfg, [w])
    outs = []
    for _ in range(2):
        dx = dev(x)
        st.forward(dx, dev(ctx))
        outs.append(host(dx))
    assert np.array_equal(outs[0], outs[1])


@pytest.mark.timeout(600)
@pytest.mark.parametrize("stage", ["A", "B"])
def test_sdxl_stage_2048_shapes_sampled_rows(hb, stage):
    """One block at the stage shapes of a 2048 x 2048 image (16384 tokens x 640, 4096 x 1280; batch 2) on
    sampled token rows."""
    from paper_2602_21760_amd import model
    cfg = synth.CFG7A if stage == "A" else synth.CFG7B
    w = synth.sdxl_block_weights(cfg, 0)
    x, ctx = synth.sdxl_inputs(cfg)
    st = model.SDXLStage(cfg, [w])
    dx = dev(x)
    st.forward(dx, dev(ctx))
    rows = np.unique(np.concatenate([[0, 127, 128, cfg.tokens - 1], np.random.default_rng(6).integers(0, cfg.tokens, 44)]))
    ref = O.sdxl_block_rows(x, ctx, w, cfg.heads, rows)
    got = host(dx)[:, rows]
    assert err(got, ref) < TOL_BF16
    assert err(got - x[:, rows], ref - x[:, rows]) < 5e-2


def test_sdxl_guidance_step(hb):
    """CFG (scale 5), both discrepancies and the Euler-epsilon update on the 128 x 128 x 4 latent; the two
    branch predictions are seeded stand-ins of the latent's shape."""
    n = int(np.prod(synth.CFG5_LATENT))
    e_c, e_u, x = synth.guidance_inputs(n, 1, "bf16", seed=55, delta=0.2)
    sig, sig_next = 14.6, 11.9
    rx, rv, r1, r2 = O.guided_step(x, e_c, e_u, synth.CFG5_GUIDANCE, np.float32(sig), np.float32(sig_next))
    dx = dev(x)
    d1, d2 = torch.empty(1, device="cuda"), torch.empty(1, device="cuda")
    ws = torch.empty(hb.hyb_discrepancy_workspace_bytes(1, n), device="cuda", dtype=torch.uint8)
    hb.hyb_cfg_disc_euler(dev(e_c, torch.bfloat16), dev(e_u, torch.bfloat16), dx, dx, synth.CFG5_GUIDANCE, sig, sig_next, d1, d2, ws)
    assert err(host(dx), rx) < 1e-6
    assert abs(d1.item() - r1[0]) < TOL_DISC * r1[0] and abs(d2.item() - r2[0]) < TOL_DISC * r2[0]
