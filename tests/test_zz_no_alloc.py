"""The allocation-free form of the fused guidance pass (hyb_cfg_disc_euler_noalloc: partial sums in a device
array built into the library) against hyb_cfg_disc_euler with a caller workspace, through the C ABI: two calls
in a row, the second on a smaller input, every output bit for bit; sizes beyond the built-in scratch are refused."""
import numpy as np
import pytest
import torch

from oracle import hyb_oracle as O
from paper_2602_21760_amd import synth
from gpu_util import TOL_DISC, dev, host, rel_l2

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hb():
    from paper_2602_21760_amd import binding
    binding.lib()
    return binding


def _both(hb, batch, n, vd, seed):
    v_c, v_u, x = synth.guidance_inputs(n, batch, vd, seed=seed)
    tdt = torch.bfloat16 if vd == "bf16" else torch.float32
    dvc, dvu, dx = dev(v_c, tdt), dev(v_u, tdt), dev(x)
    outs = []
    for form in ("workspace", "noalloc"):
        x_out, v_out = torch.empty_like(dx), torch.empty_like(dvc)
        x_lowp = torch.empty(batch, n, device="cuda", dtype=torch.bfloat16)
        d1 = torch.full((batch,), -1.0, device="cuda")
        d2 = torch.full((batch,), -1.0, device="cuda")
        if form == "workspace":
            ws = torch.empty(max(hb.hyb_discrepancy_workspace_bytes(batch, n), 256), device="cuda", dtype=torch.uint8)
            hb.hyb_cfg_disc_euler(dvc, dvu, dx, x_out, 7.0, 0.5, 0.45, d1, d2, ws, x_out_lowp=x_lowp, v_out=v_out)
        else:
            hb.hyb_cfg_disc_euler_noalloc(dvc, dvu, dx, x_out, 7.0, 0.5, 0.45, d1, d2, x_out_lowp=x_lowp, v_out=v_out)
        torch.cuda.synchronize()
        outs.append((x_out, v_out, x_lowp, d1, d2))
    ref = O.guided_step(x, v_c, v_u, 7.0, np.float32(0.5), np.float32(0.45))
    return outs, ref


def test_noalloc_matches_workspace_form_on_two_calls_in_a_row(hb):
    # first a large input (4 samples of the SD3 1024 x 1024 latent), then a smaller, ragged one: the built-in
    # array still holds the first call's partial sums when the second call runs
    for batch, n, vd, seed in ((4, 262144, "bf16", 300), (2, 4104, "f32", 301), (1, 1000, "bf16", 302)):
        (a, b), ref = _both(hb, batch, n, vd, seed)
        for ta, tb in zip(a, b):
            assert torch.equal(ta, tb)
        rx, _, r1, r2 = ref
        assert rel_l2(host(b[0]), rx) < 1e-6
        np.testing.assert_allclose(host(b[3]), r1, rtol=1e-5)
        np.testing.assert_allclose(host(b[4]), r2, rtol=1e-5)
        assert 1e-5 < TOL_DISC


def test_noalloc_rejects_sizes_beyond_the_builtin_scratch(hb):
    assert hb.hyb_discrepancy_workspace_bytes(8, 1 << 20) == 1 << 20       # exactly the built-in scratch
    n = 1 << 20
    v = torch.zeros(9, n, device="cuda", dtype=torch.bfloat16)
    x = torch.zeros(9, n, device="cuda")
    d = torch.zeros(9, device="cuda")
    with pytest.raises(hb.HybError) as e:
        hb.hyb_cfg_disc_euler_noalloc(v, v, x, x, 7.0, 0.5, 0.45, d, d)
    assert e.value.code == 5
    hb.hyb_cfg_disc_euler_noalloc(v[:8], v[:8], x[:8], x[:8], 7.0, 0.5, 0.45, d[:8], d[:8])   # the largest size that fits
    hb.hyb_cfg_disc_euler_noalloc(v, v, x, x, 7.0, 0.5, 0.45)              # no discrepancy outputs: no scratch, any size
    torch.cuda.synchronize()
    assert torch.all(d[:8] == 0)
