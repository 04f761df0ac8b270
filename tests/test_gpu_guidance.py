"""GPU parity: CFG combine, branch discrepancy, Euler update and the fused single pass, through
the C ABI, against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

from oracle import hyb_oracle as O
from paper_2602_21760_amd import synth
from gpu_util import TOL_DISC, dev, host, rel_l2, tdt

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hb():
    from paper_2602_21760_amd import binding
    binding.lib()
    return binding


def _ws(hb, batch, n):
    return torch.empty(max(hb.hyb_discrepancy_workspace_bytes(batch, n), 256), device="cuda", dtype=torch.uint8)


# sizes: scalar path with ragged tail, one partial chunk, several chunks with a tail, the real latents
SIZES = [1, 1000, 4104, 65536, 262144]


@pytest.mark.parametrize("vd", ["f32", "bf16"])
@pytest.mark.parametrize("n", SIZES)
@pytest.mark.parametrize("batch", [1, 3])
def test_fused_pass_matches_oracle(hb, vd, n, batch):
    v_c, v_u, x = synth.guidance_inputs(n, batch, vd, seed=100 + n % 97)
    s, t, t_next = 7.0, 0.5, 0.45
    ref_x, ref_v, ref_d1, ref_d2 = O.guided_step(x, v_c, v_u, s, np.float32(t), np.float32(t_next))
    dvc, dvu, dx = dev(v_c, tdt(vd)), dev(v_u, tdt(vd)), dev(x)
    x_out, v_out = torch.empty_like(dx), torch.empty_like(dvc)
    x_lowp = torch.empty(batch, n, device="cuda", dtype=torch.bfloat16)
    d1 = torch.full((batch,), -1.0, device="cuda")
    d2 = torch.full((batch,), -1.0, device="cuda")
    hb.hyb_cfg_disc_euler(dvc, dvu, dx, x_out, s, t, t_next, d1, d2, _ws(hb, batch, n), x_out_lowp=x_lowp, v_out=v_out)
    assert rel_l2(host(x_out), ref_x) < 1e-6
    assert rel_l2(host(v_out), ref_v) < (4e-3 if vd == "bf16" else 1e-6)     # bf16 output rounding of v only
    assert rel_l2(host(x_lowp), ref_x) < 4e-3
    np.testing.assert_allclose(host(d1), ref_d1, rtol=1e-5)
    np.testing.assert_allclose(host(d2), ref_d2, rtol=1e-5)
    assert 1e-5 < TOL_DISC
    # in place (x_out aliases x), optional outputs skipped
    hb.hyb_cfg_disc_euler(dvc, dvu, dx, dx, s, t, t_next)
    assert rel_l2(host(dx), ref_x) < 1e-6


@pytest.mark.parametrize("vd", ["f32", "bf16"])
def test_separate_calls_match_oracle(hb, vd):
    n, batch = 70001, 2
    v_c, v_u, x = synth.guidance_inputs(n, batch, vd, seed=7)
    dvc, dvu, dx = dev(v_c, tdt(vd)), dev(v_u, tdt(vd)), dev(x)
    v = torch.empty_like(dvc)
    hb.hyb_cfg_combine(dvc, dvu, v, 5.0)
    assert rel_l2(host(v), O.cfg_combine(v_c, v_u, 5.0)) < (4e-3 if vd == "bf16" else 1e-6)
    out = torch.empty(batch, device="cuda")
    for p in (1, 2):
        hb.hyb_branch_discrepancy(dvc, dvu, p, out, _ws(hb, batch, n))
        np.testing.assert_allclose(host(out), O.branch_discrepancy(v_c, v_u, p), rtol=1e-5)
    xo = torch.empty_like(dx)
    hb.hyb_euler_step(dx, dvc, xo, 0.5, 0.45)
    assert rel_l2(host(xo), O.euler_step(x, v_c, np.float32(0.5), np.float32(0.45))) < 1e-6
    # bf16 latent variant
    xb = dx.to(torch.bfloat16)
    xbo = torch.empty_like(xb)
    hb.hyb_euler_step(xb, dvc, xbo, 1.0, 0.0)
    assert rel_l2(host(xbo), O.euler_step(host(xb), v_c, 1.0, 0.0)) < 4e-3


def test_closed_forms_on_gpu(hb):
    n = 8192 + 24
    v_c, v_u, x = synth.guidance_inputs(n, 1, "bf16", seed=3)
    dvc, dvu, dx = dev(v_c, torch.bfloat16), dev(v_u, torch.bfloat16), dev(x)
    v = torch.empty_like(dvc)
    hb.hyb_cfg_combine(dvc, dvu, v, 0.0)
    assert torch.equal(v, dvu)                                   # scale 0 -> unconditional, exactly
    hb.hyb_cfg_combine(dvc, dvu, v, 1.0)
    assert rel_l2(host(v), v_c) < 1e-6                           # scale 1 -> conditional
    hb.hyb_cfg_combine(dvu, dvu, v, 7.0)
    assert torch.equal(v, dvu)                                   # equal branches -> unchanged for any scale
    d1, d2 = torch.full((1,), -1.0, device="cuda"), torch.full((1,), -1.0, device="cuda")
    ws = _ws(hb, 1, n)
    xo = torch.empty_like(dx)
    hb.hyb_cfg_disc_euler(dvu, dvu, dx, xo, 7.0, 0.3, 0.3, d1, d2, ws)
    assert d1.item() == 0.0 and d2.item() == 0.0                 # equal branches -> discrepancy 0
    assert torch.equal(xo, dx)                                   # t_next == t -> identity
    z = torch.zeros_like(dvu)
    hb.hyb_cfg_disc_euler(dvc, z, dx, xo, 7.0, 0.3, 0.2, d1, d2, ws)
    assert d1.item() == float("inf") and d2.item() == float("inf")
    hb.hyb_cfg_disc_euler(z, z, dx, xo, 7.0, 0.3, 0.2, d1, d2, ws)
    assert d1.item() == 0.0 and d2.item() == 0.0
    # v_c = (1 + a) v_u -> |a| for both norms (a = 0.5 keeps bf16 values exact)
    hb.hyb_cfg_disc_euler((dvu.float() * 1.5).to(torch.bfloat16), dvu, dx, xo, 7.0, 0.3, 0.2, d1, d2, ws)
    ref = O.branch_discrepancy(host((dvu.float() * 1.5).to(torch.bfloat16)), v_u, 1)[0]
    assert abs(d1.item() - ref) < 1e-5 * ref and abs(d1.item() - 0.5) < 2e-3 and abs(d2.item() - 0.5) < 2e-3


def test_affine_update_and_batch_invariance(hb):
    n = 262144
    v_c, v_u, x = synth.guidance_inputs(n, 1, "bf16", seed=5)
    # the same sample at batch index 0 and 2, a different one in between
    o_c, o_u, o_x = synth.guidance_inputs(n, 1, "bf16", seed=6)
    stack = lambda a, b: np.concatenate([a, b, a])
    dvc, dvu, dx = dev(stack(v_c, o_c), torch.bfloat16), dev(stack(v_u, o_u), torch.bfloat16), dev(stack(x, o_x))
    xo = torch.empty_like(dx)
    d1, d2 = torch.empty(3, device="cuda"), torch.empty(3, device="cuda")
    a, b = 0.98, -0.07
    hb.hyb_cfg_disc_affine(dvc, dvu, dx, xo, 5.0, a, b, d1, d2, _ws(hb, 3, n))
    ref = O.affine_step(x, O.cfg_combine(v_c, v_u, 5.0), np.float32(a), np.float32(b))
    assert rel_l2(host(xo[0:1]), ref) < 1e-6
    assert torch.equal(xo[0], xo[2]) and d1[0].item() == d1[2].item() and d2[0].item() == d2[2].item()
    assert d1[0].item() != d1[1].item()
    # run-to-run determinism
    xo2, e1, e2 = torch.empty_like(dx), torch.empty(3, device="cuda"), torch.empty(3, device="cuda")
    hb.hyb_cfg_disc_affine(dvc, dvu, dx, xo2, 5.0, a, b, e1, e2, _ws(hb, 3, n))
    assert torch.equal(xo, xo2) and torch.equal(d1, e1) and torch.equal(d2, e2)


def test_empty_inputs_and_errors(hb):
    e = torch.empty(0, device="cuda")
    hb.hyb_cfg_combine(e, e, e, 3.0)
    hb.hyb_euler_step(e, e, e, 0.5, 0.4)
    d = torch.full((2,), -1.0, device="cuda")
    e2 = torch.empty(2, 0, device="cuda")
    hb.hyb_branch_discrepancy(e2, e2, 2, d, None)      # empty samples: 0 / 0 -> 0
    assert host(d).tolist() == [0.0, 0.0]
    v = torch.zeros(1, 4096, device="cuda")
    with pytest.raises(hb.HybError) as ei:
        hb.hyb_branch_discrepancy(v, v, 2, d, torch.empty(16, device="cuda", dtype=torch.uint8))
    assert ei.value.code == 5
    with pytest.raises(hb.HybError) as ei:
        hb.hyb_branch_discrepancy(v, v, 2, d, None)
    assert ei.value.code == 1
