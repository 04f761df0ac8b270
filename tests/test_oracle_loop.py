"""Pins for the oracle's guided sampling loop (Alg. 1 without the stage switch; CFG of Sec. 3; flow ODE of
Sec. 3 integrated from t = 1 to t = 0) and for the two small modulation helpers, by cases whose result is
known without running the loop: a branch the guidance scale switches off cannot matter, a constant velocity
field integrates to x_0 - v over the whole schedule, equal branches have zero discrepancy, and one step of
the loop is the composition of the pinned single-step functions."""
import numpy as np
import torch
import torch.nn.functional as F

from oracle import hyb_oracle as O
from paper_2602_21760_amd import synth


def _setup(blocks=1, scale=10.0):
    cfg = synth.scaled(synth.CFG1, blocks=blocks, hidden=128, heads=2, latent_hw=8, latent_c=4, n_txt=5,
                       ctx_dim=32, batch=1)
    P = {n: a * scale for n, a in synth.mmdit_globals(cfg).items()}
    P["pos"] = P["pos"] / scale
    bl = [{s: {n: a * scale for n, a in d.items()} for s, d in synth.mmdit_block_weights(cfg, i).items()}
          for i in range(cfg.blocks)]
    lat, ctx_c, ctx_u = synth.mmdit_inputs(cfg)
    return cfg, P, bl, lat[None], ctx_c[None], ctx_u[None]


def test_loop_ignores_the_branch_the_scale_switches_off():
    cfg, P, bl, lat, ctx_c, ctx_u = _setup()
    other = np.random.default_rng(5).standard_normal(ctx_u.shape)
    # s = 1: conditional prediction only (Sec. 3, w = 0)
    xa, _, _ = O.sampling_loop(lat, ctx_c, ctx_u, P, lambda: bl, cfg.heads, cfg.patch, 3, 3.0, 1.0)
    xb, _, _ = O.sampling_loop(lat, ctx_c, other, P, lambda: bl, cfg.heads, cfg.patch, 3, 3.0, 1.0)
    np.testing.assert_allclose(xa, xb, rtol=1e-10, atol=1e-12)
    # s = 0: unconditional prediction only
    xc, _, _ = O.sampling_loop(lat, ctx_c, ctx_u, P, lambda: bl, cfg.heads, cfg.patch, 3, 3.0, 0.0)
    xd, _, _ = O.sampling_loop(lat, other, ctx_u, P, lambda: bl, cfg.heads, cfg.patch, 3, 3.0, 0.0)
    np.testing.assert_allclose(xc, xd, rtol=1e-10, atol=1e-12)
    assert np.abs(xa - xc).max() > 1e-6     # and the text does matter otherwise


def test_loop_with_constant_velocity_integrates_to_x_minus_v():
    cfg, P, bl, lat, ctx_c, ctx_u = _setup()
    P["f_w"] = np.zeros_like(P["f_w"])      # v = unpatchify(b_f) whatever the tokens, the text and the time are
    v = O.unpatchify(np.broadcast_to(P["f_b"], (1, cfg.n_img, P["f_b"].shape[0])), cfg.latent_hw, cfg.latent_hw,
                     cfg.latent_c, cfg.patch)
    for T_steps, shift in ((1, 3.0), (4, 3.0), (5, 1.0)):
        x, M1, M2 = O.sampling_loop(lat, ctx_c, ctx_u, P, lambda: bl, cfg.heads, cfg.patch, T_steps, shift, 7.0)
        np.testing.assert_allclose(x, lat - v, rtol=1e-12, atol=1e-12)     # sum of the steps' dt is 0 - 1
        assert M1.shape == (T_steps, 1) and M2.shape == (T_steps, 1)
        assert np.all(M1 == 0) and np.all(M2 == 0)                          # equal branches: Eq. 1 gives 0


def test_loop_step_is_the_composition_of_the_single_step_functions():
    cfg, P, bl, lat, ctx_c, ctx_u = _setup(blocks=2)
    T_steps, shift, s = 2, 3.0, 7.0
    x, M1, M2 = O.sampling_loop(lat, ctx_c, ctx_u, P, lambda: bl, cfg.heads, cfg.patch, T_steps, shift, s)
    sig = [1.0, 3.0 * 0.5 / (1.0 + 2.0 * 0.5), 0.0]      # closed form of the shifted schedule at u = 1, 1/2, 0
    xr = lat.astype(np.float64)
    for i in range(T_steps):
        t = np.array([sig[i]])
        v_c = O.mmdit_forward(xr, ctx_c, t, P, bl, cfg.heads, cfg.patch)
        v_u = O.mmdit_forward(xr, ctx_u, t, P, bl, cfg.heads, cfg.patch)
        d = v_c - v_u
        np.testing.assert_allclose(M1[i, 0], np.abs(d).sum() / np.abs(v_u).sum(), rtol=1e-12)
        np.testing.assert_allclose(M2[i, 0], np.sqrt((d * d).sum() / (v_u * v_u).sum()), rtol=1e-12)
        xr = xr + (sig[i + 1] - sig[i]) * (v_c + (s - 1.0) * d)     # the paper's eps_c + w (eps_c - eps_u), w = s - 1
    np.testing.assert_allclose(x, xr, rtol=1e-10, atol=1e-12)
    assert M1[0, 0] > 0


def test_modulate_special_cases():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((2, 5, 8))
    sh, sc = rng.standard_normal((2, 8)), rng.standard_normal((2, 8))
    zero = np.zeros((2, 8))
    np.testing.assert_array_equal(O.modulate(x, zero, zero), x)
    # scale = -1 removes the input: what is left is the shift, the same for every token
    np.testing.assert_allclose(O.modulate(x, sh, -np.ones((2, 8))), np.broadcast_to(sh[:, None, :], x.shape), atol=1e-15)
    # scale = 1 doubles, per sample and feature
    np.testing.assert_allclose(O.modulate(x, zero, np.ones((2, 8))), 2 * x, rtol=1e-15)
    # affine in each argument
    np.testing.assert_allclose(O.modulate(x, sh, sc) - O.modulate(x, zero, sc), np.broadcast_to(sh[:, None, :], x.shape),
                               rtol=1e-12, atol=1e-12)
    a = O.modulate(x, sh, sc)
    assert not np.allclose(a[0], a[1] - x[1] + x[0])     # the two samples use their own rows of shift / scale


def test_adaln_modulation_chunks():
    rng = np.random.default_rng(1)
    D = 6
    temb = rng.standard_normal((3, D))
    b = rng.standard_normal(6 * D)
    # zero weights: the chunks are the six slices of the bias, in order, for every sample
    parts = O.adaln_modulation(temb, np.zeros((6 * D, D)), b, 6)
    assert len(parts) == 6
    for kk, part in enumerate(parts):
        np.testing.assert_array_equal(part, np.broadcast_to(b[kk * D:(kk + 1) * D], (3, D)))
    # stacked multiples of the identity: chunk kk is (kk + 1) SiLU(temb), with the library's SiLU
    W = np.concatenate([(kk + 1) * np.eye(D) for kk in range(6)], axis=0)
    parts = O.adaln_modulation(temb, W, np.zeros(6 * D), 6)
    ref = F.silu(torch.from_numpy(temb)).numpy()
    for kk, part in enumerate(parts):
        np.testing.assert_allclose(part, (kk + 1) * ref, rtol=1e-13)
    assert len(O.adaln_modulation(temb, W[:2 * D], np.zeros(2 * D), 2)) == 2
