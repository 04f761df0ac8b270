"""GPU parity of the denoiser building blocks (linear + epilogues, LayerNorm-modulate, adaLN
modulation, timestep features, patchify, attention) against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import hyb_oracle as O
from paper_2602_21760_amd import synth
from gpu_util import dev, host, err, tdt, tol

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hb():
    from paper_2602_21760_amd import binding
    binding.lib()
    return binding


def _data(seed, shape, dt, std=1.0):
    return synth.normal(seed, shape, std, dt)


# (m, n, k): ragged rows, several tiles, the real GEMM shapes' aspect; k a multiple of 64 for the MFMA
# path, an odd k for the plain kernel (f32 only).  The MFMA kernel uses 64-row tiles for grids of at most 384
# 128-row tiles and 128-row tiles beyond: the last shape (9 x 44 = 396 tiles, ragged both ways) takes the latter.
LINEAR_SHAPES = [(1, 64, 64), (77, 128, 64), (333, 1536, 256), (300, 72, 128), (513, 384, 192), (1100, 5576, 128)]


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("shape", LINEAR_SHAPES)
def test_linear_epilogues(hb, dt, shape):
    m, n, k = shape
    a, w, b = _data(1, (m, k), dt), _data(2, (n, k), dt, 0.05), _data(3, (n,), "f32", 0.5)
    da, dw, db = dev(a, tdt(dt)), dev(w, tdt(dt)), dev(b)
    y = O.linear(a, w, b)
    for epi, fn in ((hb.HYB_EPI_BIAS, lambda z: z), (hb.HYB_EPI_GELU_TANH, O.gelu_tanh), (hb.HYB_EPI_SILU, O.silu)):
        for od in ("f32", dt):
            out = torch.empty(m, n, device="cuda", dtype=tdt(od))
            hb.hyb_linear(da, dw, db, out, epi)
            assert err(host(out), fn(y)) < (tol(dt) if od == "f32" and dt == "f32" else max(tol(dt), 4e-3))
    # gate * y + residual with a per-sample gate (3 "samples" of ragged size) and without gate
    rpg = (m + 2) // 3
    res, gate = _data(4, (m, n), "f32"), _data(5, (3, 2 * n), "f32")
    dres, dgate = dev(res), dev(gate)
    out = torch.empty(m, n, device="cuda")
    hb.hyb_linear(da, dw, db, out, hb.HYB_EPI_GATE_RESIDUAL, residual=dres, gate=dgate[:, n:], rows_per_gate=rpg,
                  gate_stride=2 * n)
    g_rows = gate[np.arange(m) // rpg, n:]
    assert err(host(out), res + g_rows * y) < tol(dt)
    hb.hyb_linear(da, dw, db, dres, hb.HYB_EPI_GATE_RESIDUAL, residual=dres)     # in place, gate = 1
    assert err(host(dres), res + y) < tol(dt)
    # no bias
    out = torch.empty(m, n, device="cuda")
    hb.hyb_linear(da, dw, None, out)
    assert err(host(out), O.linear(a, w)) < tol(dt)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(77, 64, 64), (333, 200, 128), (1100, 2560, 192), (45, 37, 24)])
def test_linear_geglu(hb, dt, shape):
    """out = (a Wu^T + bu) * GELUerf(a Wg^T + bg), W = [Wu; Wg]: the gated feed-forward projection of the
    SDXL-shaped block through the public entry point (MFMA kernel for bf16 with k % 64 == 0, plain kernel else)."""
    m, n, k = shape
    a, w, b = _data(1, (m, k), dt), _data(2, (2 * n, k), dt, 0.08), _data(3, (2 * n,), "f32", 0.5)
    da, dw, db = dev(a, tdt(dt)), dev(w, tdt(dt)), dev(b)
    ref = O.linear(a, w[:n], b[:n]) * O.gelu_erf(O.linear(a, w[n:], b[n:]))
    for od in ("f32", dt):
        out = torch.empty(m, n, device="cuda", dtype=tdt(od))
        hb.hyb_linear(da, dw, db, out, hb.HYB_EPI_GEGLU)
        assert err(host(out), ref) < (tol(dt) if od == "f32" and dt == "f32" else max(tol(dt), 4e-3))
    out = torch.empty(m, n, device="cuda", dtype=tdt(dt))
    hb.hyb_linear(da, dw, None, out, hb.HYB_EPI_GEGLU)                       # no bias
    assert err(host(out), O.linear(a, w[:n]) * O.gelu_erf(O.linear(a, w[n:]))) < max(tol(dt), 4e-3)


def test_linear_odd_k_f32(hb):
    m, n, k = 45, 37, 19
    a, w, b = _data(1, (m, k), "f32"), _data(2, (n, k), "f32"), _data(3, (n,), "f32")
    out = torch.empty(m, n, device="cuda")
    hb.hyb_linear(dev(a), dev(w), dev(b), out)
    assert err(host(out), O.linear(a, w, b)) < 1e-6


@pytest.mark.parametrize("od", ["f32", "bf16"])
@pytest.mark.parametrize("hidden", [256, 1536, 2048, 640])
def test_layernorm_modulate(hb, od, hidden):
    B, T = 2, 37
    x = _data(10, (B, T, hidden), "f32") * 3 + 0.5
    mod = _data(11, (B, 3 * hidden), "f32", 0.3)
    dx, dmod = dev(x), dev(mod)
    out = torch.empty(B, T, hidden, device="cuda", dtype=tdt(od))
    hb.hyb_layernorm_modulate(dx, dmod[:, hidden:], dmod[:, 2 * hidden:], 3 * hidden, out, 1e-6)
    ref = O.modulate(O.layer_norm(x, 1e-6), mod[:, hidden:2 * hidden], mod[:, 2 * hidden:])
    assert err(host(out), ref) < (4e-3 if od == "bf16" else 1e-5)
    hb.hyb_layernorm_modulate(dx, None, None, 0, out, 1e-6)
    assert err(host(out), O.layer_norm(x, 1e-6)) < (4e-3 if od == "bf16" else 1e-5)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("batch", [1, 2, 5])
def test_adaln_modulation(hb, dt, batch):
    rows, hidden = 6 * 256 + 10, 256
    w, b = _data(20, (rows, hidden), dt, 0.05), _data(21, (rows,), "f32")
    temb = _data(22, (batch, hidden), "f32")
    out = torch.empty(batch, rows, device="cuda")
    hb.hyb_adaln_modulation(dev(w, tdt(dt)), dev(b), dev(temb), out)
    assert err(host(out), O.linear(O.silu(temb), w, b)) < 1e-5


def test_timestep_embedding_and_patchify(hb):
    t = np.array([0.0, 0.5, 0.45, 1.0], dtype=np.float32)
    out = torch.empty(4, 256, device="cuda")
    hb.hyb_timestep_embedding(dev(t), out)
    np.testing.assert_allclose(host(out), O.timestep_embedding(t, 256), atol=2e-7)
    lat = _data(30, (2, 16, 12, 4), "f32")
    tok = torch.empty(2, 8 * 6, 16, device="cuda")
    hb.hyb_patchify(dev(lat), tok, 2)
    np.testing.assert_array_equal(host(tok), O.patchify(lat, 2))
    back = torch.empty(2, 16, 12, 4, device="cuda")
    hb.hyb_unpatchify(tok, back, 2)
    np.testing.assert_array_equal(host(back), lat.astype(np.float64))
    tokb = torch.empty(2, 8 * 6, 16, device="cuda", dtype=torch.bfloat16)
    hb.hyb_patchify(dev(lat), tokb, 2)
    np.testing.assert_array_equal(host(tokb), O.patchify(synth.round_bf16(lat), 2))
    c = torch.empty(2 * 16 * 12 * 4, device="cuda", dtype=torch.bfloat16)
    hb.hyb_convert(dev(lat).view(-1), c)
    np.testing.assert_array_equal(host(c), synth.round_bf16(lat).reshape(-1).astype(np.float64))


# (batch, heads, n_q, n_kv): tiny, exactly one tile, tile + 1, ragged joint sizes (image + 333 text
# tokens), cross-attention to 77 keys
ATTN_SHAPES = [(1, 1, 1, 1), (2, 2, 64, 64), (1, 3, 65, 65), (2, 2, 80, 80), (1, 2, 461, 461), (2, 2, 200, 77),
               (1, 1, 130, 333)]


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("shape", ATTN_SHAPES)
def test_attention(hb, dt, shape):
    B, H, Nq, Nk = shape
    q, k, v = _data(40, (B, H, Nq, 64), dt), _data(41, (B, H, Nk, 64), dt), _data(42, (B, H, Nk, 64), dt)
    o = torch.empty(B, Nq, H * 64, device="cuda", dtype=tdt(dt))
    hb.hyb_joint_attention(dev(q, tdt(dt)), dev(k, tdt(dt)), dev(v, tdt(dt)), o)
    assert err(host(o), O.attention(q, k, v)) < (tol(dt) if dt == "f32" else 1e-2)
    hb.hyb_joint_attention(dev(q, tdt(dt)), dev(k, tdt(dt)), dev(v, tdt(dt)), o, scale=0.3)
    assert err(host(o), O.attention(q, k, v, scale=0.3)) < (tol(dt) if dt == "f32" else 1e-2)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_attention_invariants_on_gpu(hb, dt):
    B, H, N = 1, 2, 150
    q, v = _data(50, (B, H, N, 64), dt), _data(51, (B, H, N, 64), dt)
    k = np.repeat(_data(52, (B, H, 1, 64), dt), N, axis=2)           # all keys equal -> mean of V
    o = torch.empty(B, N, H * 64, device="cuda", dtype=tdt(dt))
    hb.hyb_joint_attention(dev(q, tdt(dt)), dev(k, tdt(dt)), dev(v, tdt(dt)), o)
    mean_v = np.concatenate([v[0, h].astype(np.float64).mean(0) for h in range(H)])
    assert err(host(o)[0], np.broadcast_to(mean_v, (N, H * 64))) < (1e-5 if dt == "f32" else 1e-2)
    # large logits: the streaming softmax must not overflow
    # (scaled by a power of two: the scaled values stay bf16-representable, so both sides see the same data)
    qb = _data(53, (B, H, N, 64), dt) * 8
    kb = _data(54, (B, H, N, 64), dt) * 4
    hb.hyb_joint_attention(dev(qb, tdt(dt)), dev(kb, tdt(dt)), dev(v, tdt(dt)), o)
    got = host(o)
    assert np.isfinite(got).all()
    assert err(got, O.attention(qb, kb, v)) < (1e-4 if dt == "f32" else 1e-2)


@pytest.mark.parametrize("growth", [3.0, 7.5, 40.0])
def test_attention_running_maximum_schedules(hb, growth):
    """Scores that rise steadily along the key axis: the row maximum of every 64-key tile exceeds the previous
    one by `growth` (in base-2 exponent units), so the kernel's deferred rescaling (it only advances its running
    maximum when the tile maximum has grown by more than 2^8) sees growth below, just below and far above its
    threshold; descending order (the first tile holds the maximum) rides along as the second head.  All scores sit
    2^80 above zero, so that the kernel's first attempt (sums without a reference maximum) is out of range for every
    row and the loop with the running maximum is what produces the result."""
    B, H, N = 1, 2, 650                               # 10 full tiles + a ragged one
    rng = np.random.default_rng(77)
    q = np.zeros((B, H, N, 64), np.float32)
    k = np.zeros((B, H, N, 64), np.float32)
    q[..., 0] = 8.0
    # score_j * log2(e) = 80 + growth * j / 64
    ramp = (80.0 + growth / 64.0 * np.arange(N)) / (8.0 * 0.125 * 1.4426950408889634)
    k[0, 0, :, 0] = ramp
    k[0, 1, :, 0] = ramp[::-1]
    q[..., 1:] = synth.round_bf16(0.05 * rng.standard_normal((B, H, N, 63)).astype(np.float32))
    k[..., 1:] = synth.round_bf16(0.05 * rng.standard_normal((B, H, N, 63)).astype(np.float32))
    k = synth.round_bf16(k)
    v = _data(78, (B, H, N, 64), "bf16")
    o = torch.empty(B, N, H * 64, device="cuda", dtype=torch.bfloat16)
    hb.hyb_joint_attention(dev(q, torch.bfloat16), dev(k, torch.bfloat16), dev(v, torch.bfloat16), o)
    got = host(o)
    assert np.isfinite(got).all()
    assert err(got, O.attention(q, k, v)) < 1e-2


@pytest.mark.parametrize("shape", [(1, 8, 5118, 5118), (1, 8, 700, 700), (2, 12, 4429, 4429)])
def test_attention_with_workspace_splits_and_matches(hb, shape):
    """hyb_joint_attention_ws: with scratch the kernel may cut overloading query blocks along the keys and merge
    the parts; both forms against the oracle (sampled rows incl. the last query blocks, which are the ones that
    get cut), the two forms against each other, and the split form twice for identical bits."""
    B, H, Nq, Nk = shape
    q, k, v = _data(140, (B, H, Nq, 64), "bf16"), _data(141, (B, H, Nk, 64), "bf16"), _data(142, (B, H, Nk, 64), "bf16")
    dq, dk, dv = (dev(a, torch.bfloat16) for a in (q, k, v))
    need = hb.hyb_joint_attention_workspace_bytes(B, H, Nq, hb.HYB_BF16)
    assert (need > 0) == (Nq != 700)                  # 6 query blocks per XCD never overload a CU
    ws = torch.empty(max(need, 256), device="cuda", dtype=torch.uint8)
    o_ws, o_ws2, o_plain = (torch.empty(B, Nq, H * 64, device="cuda", dtype=torch.bfloat16) for _ in range(3))
    hb.hyb_joint_attention_ws(dq, dk, dv, o_ws, ws)
    ws.fill_(0xFF)                                    # contents of the scratch are irrelevant on entry
    hb.hyb_joint_attention_ws(dq, dk, dv, o_ws2, ws)
    hb.hyb_joint_attention(dq, dk, dv, o_plain)
    assert torch.equal(o_ws, o_ws2)
    rows = np.unique(np.concatenate([np.arange(Nq - 200, Nq), [0, 1, 127, 128], np.random.default_rng(3).integers(0, Nq, 60)]))
    ref = O.attention(q, k, v, rows=rows)
    assert err(host(o_ws)[:, rows], ref) < 1e-2 and err(host(o_plain)[:, rows], ref) < 1e-2
    assert err(host(o_ws), host(o_plain)) < 1e-2      # every row of the two forms (bf16 output rounding apart)
    if need == 0:
        assert torch.equal(o_ws, o_plain)
    if need:
        with pytest.raises(hb.HybError):
            hb.hyb_joint_attention_ws(dq, dk, dv, o_ws, ws[:need - 256])


LN2 = 0.6931471805599453


def _prescaled(hb, q, k, v, dt="bf16", fill=None):
    B, H, Nq, _ = q.shape
    need = hb.hyb_joint_attention_workspace_bytes(B, H, Nq, hb.HYB_BF16 if dt == "bf16" else hb.HYB_F32)
    ws = torch.empty(max(need, 256), device="cuda", dtype=torch.uint8)
    if fill is not None:
        ws.fill_(fill)
    o = torch.empty(B, Nq, H * 64, device="cuda", dtype=tdt(dt))
    hb.hyb_joint_attention_prescaled(dev(q, tdt(dt)), dev(k, tdt(dt)), dev(v, tdt(dt)), o, ws)
    return o


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("shape", ATTN_SHAPES)
def test_attention_prescaled(hb, dt, shape):
    """Queries that already hold scale x log2(e): the result is the base-2 softmax of q k^T, i.e. the oracle's
    attention with scale = ln 2.  Scores of a few units: the bf16 kernel's sums without a reference maximum."""
    B, H, Nq, Nk = shape
    q, k, v = _data(240, (B, H, Nq, 64), dt, 0.2), _data(241, (B, H, Nk, 64), dt), _data(242, (B, H, Nk, 64), dt)
    got = host(_prescaled(hb, q, k, v, dt))
    assert err(got, O.attention(q, k, v, scale=LN2)) < (tol(dt) if dt == "f32" else 1e-2)


@pytest.mark.parametrize("case", ["overflow", "underflow", "some_rows", "edge_of_range"])
def test_attention_prescaled_out_of_range_sums_start_over(hb, case):
    """Row sums of 2^score outside [2^-64, 2^64] make a workgroup start over with the running maximum: scores of
    hundreds (every row), scores near -130 (every term underflows), a few huge rows inside otherwise moderate
    128-row blocks, and sums a little inside / outside the accepted range on both sides."""
    B, H, N = 1, 2, 461
    q, k, v = _data(250, (B, H, N, 64), "bf16", 0.2), _data(251, (B, H, N, 64), "bf16"), _data(252, (B, H, N, 64), "bf16")
    if case == "overflow":
        q, k = q * 32, k * 4
    elif case == "underflow":
        q[..., 0], k[..., 0] = -16.0, 8.0 + 0.25 * np.round(k[..., 0])
    elif case == "some_rows":
        q[0, 0, 130:140] *= 64
        q[0, 1, 300] *= 256
        q[0, 1, 460, 0], k[0, 1, :, 0] = -32.0, 4.0
    else:
        # head 0: row r gets the constant (r - 230) / 2.8 added to all its scores: sums from about 2^-73 to 2^91
        k[0, 0, :, 0] = 8.0
        q[0, 0, :, 0] = synth.round_bf16(((np.arange(N) - 230) / 2.8 / 8).astype(np.float32))
    o1 = _prescaled(hb, q, k, v)
    got = host(o1)
    assert np.isfinite(got).all()
    want = O.attention(q, k, v, scale=LN2)
    assert err(got, want) < 1e-2
    assert torch.equal(o1, _prescaled(hb, q, k, v))
    # the entry point that takes the scale (here ln 2: the same scores) tries sums without a reference maximum first
    # as well, multiplying every score by scale x log2(e), and starts over in the same cases
    o2 = torch.empty_like(o1)
    hb.hyb_joint_attention(*(dev(a, torch.bfloat16) for a in (q, k, v)), o2, scale=LN2)
    got2 = host(o2)
    assert np.isfinite(got2).all()
    assert err(got2, want) < 1e-2


def test_attention_prescaled_split_parts_with_mixed_references(hb):
    """The shape whose last query blocks are cut along the keys: the first thousand keys of half the heads give
    scores of hundreds, so the key parts that hold them start over (reference = row maximum) while the other parts
    of the same rows keep reference 0, and the merge has to bring both onto one scale; the other heads stay
    moderate throughout.  Sampled rows against the oracle, all rows against the form with the scale passed in,
    twice for identical bits with the scratch overwritten in between."""
    B, H, N = 1, 8, 5118
    q, k, v = _data(260, (B, H, N, 64), "bf16", 0.2), _data(261, (B, H, N, 64), "bf16"), _data(262, (B, H, N, 64), "bf16")
    k[0, :4, :1000] *= 32
    o1 = _prescaled(hb, q, k, v)
    o2 = _prescaled(hb, q, k, v, fill=0xFF)
    assert torch.equal(o1, o2)
    rows = np.unique(np.concatenate([np.arange(N - 300, N), [0, 1, 127, 128], np.random.default_rng(5).integers(0, N, 40)]))
    assert err(host(o1)[:, rows], O.attention(q, k, v, rows=rows, scale=LN2)) < 1e-2
    need = hb.hyb_joint_attention_workspace_bytes(B, H, N, hb.HYB_BF16)
    ws = torch.empty(need, device="cuda", dtype=torch.uint8)
    o3 = torch.empty_like(o1)
    hb.hyb_joint_attention_ws(*(dev(a, torch.bfloat16) for a in (q, k, v)), o3, ws, scale=LN2)
    assert err(host(o1), host(o3)) < 1e-2


def test_workload_gemms_take_the_mfma_path(hb):
    """Every bf16 GEMM shape of the SD3-shaped and SDXL-shaped workloads (k % 64 == 0, n % 8 == 0) is served by
    the MFMA kernel: the library's launch trace names the kernel each call ran, and none is the plain FMA one."""
    shapes = {(4608, 1536), (1536, 1536), (6144, 1536), (1536, 6144), (1536, 64), (1536, 4096), (64, 1536),
              (1536, 256),                                                        # SD3-shaped branch incl. embed / final
              (1920, 640), (640, 640), (1280, 2048), (5120, 640), (640, 2560),   # SDXL stage A
              (3840, 1280), (1280, 1280), (2560, 2048), (10240, 1280), (1280, 5120)}   # stage B
    hb.hyb_trace_enable(True)
    try:
        for n, k in sorted(shapes):
            for m in (1, 77, 333, 1024):
                a = torch.zeros(m, k, device="cuda", dtype=torch.bfloat16)
                w = torch.zeros(n, k, device="cuda", dtype=torch.bfloat16)
                out = torch.empty(m, n, device="cuda", dtype=torch.bfloat16)
                hb.hyb_linear(a, w, None, out)
        torch.cuda.synchronize()
        names = hb.hyb_trace_summary()
    finally:
        hb.hyb_trace_enable(False)
    assert names and all(nm.startswith(("gemm_mfma", "gemm_splitk")) for nm in names), sorted(names)
    assert sum(r["launches"] for nm, r in names.items() if nm.startswith("gemm_mfma")) == len(shapes) * 4


@pytest.mark.parametrize("k", [3136, 3200, 3264])
def test_linear_large_tile_slab_count_remainders(hb, k):
    """The large-tile kernel's pipeline ends in three, four or five slabs outside its steady-state loop
    (49, 50, 51 k-slabs here): against the oracle, and the same bits as the 128 x 128 kernel on the first rows."""
    m, n = 2816, 1536
    a, w, b = _data(210 + k, (m, k), "bf16"), _data(211 + k, (n, k), "bf16", 0.02), _data(212, (n,), "f32", 0.02)
    da, dw, db = dev(a, torch.bfloat16), dev(w, torch.bfloat16), dev(b)
    out = torch.empty(m, n, device="cuda", dtype=torch.float32)
    hb.hyb_trace_enable(True)
    hb.hyb_linear(da, dw, db, out)
    torch.cuda.synchronize()
    names = hb.hyb_trace_summary()
    hb.hyb_trace_enable(False)
    assert list(names) == ["gemm_mfma_256x128.epi%d.n%d.k%d" % (hb.HYB_EPI_BIAS, n, k)], names
    assert err(host(out), O.linear(a, w, b)) < 1e-4
    small = torch.empty(100, n, device="cuda", dtype=torch.float32)
    hb.hyb_linear(da[:100], dw, db, small)
    assert torch.equal(out[:100], small)


def test_linear_large_tile_path(hb):
    """Long-k launches with enough 256 x 128 tiles take the large-tile kernel (the SD3-shaped fc2).  Every
    epilogue it has, ragged rows (4429 = 17 x 256 + 77) and columns (1544 = 12 x 128 + 8), gate rows that change inside
    a tile, against the oracle; the launch trace names the kernel; and, because both kernels accumulate in the same
    order, the first rows computed alone by the 128 x 128 kernel have the same bits."""
    m, n, k = 4429, 1544, 3072
    a, w, b = _data(200, (m, k), "bf16"), _data(201, (n, k), "bf16", 0.02), _data(202, (n,), "f32", 0.02)
    res, gate = _data(203, (m, n), "f32"), _data(204, (3, n), "f32")
    da, dw, db = dev(a, torch.bfloat16), dev(w, torch.bfloat16), dev(b)
    y = O.linear(a, w, b)
    g_rows = gate[np.minimum(np.arange(m) // 1500, 2)]
    cases = [("bias bf16", torch.bfloat16, hb.HYB_EPI_BIAS, {}, y, 4e-3),
             ("bias f32", torch.float32, hb.HYB_EPI_BIAS, {}, y, 1e-4),
             ("gelu", torch.bfloat16, hb.HYB_EPI_GELU_TANH, {}, O.gelu_tanh(y), 4e-3),
             ("silu", torch.bfloat16, hb.HYB_EPI_SILU, {}, O.silu(y), 4e-3),
             ("gate + residual", torch.float32, hb.HYB_EPI_GATE_RESIDUAL,
              dict(residual=dev(res), gate=dev(gate), rows_per_gate=1500, gate_stride=n), res + g_rows * y, 1e-4)]
    for name, odt, epi, kw, ref, bound in cases:
        out = torch.empty(m, n, device="cuda", dtype=odt)
        hb.hyb_trace_enable(True)
        hb.hyb_linear(da, dw, db, out, epi, **kw)
        torch.cuda.synchronize()
        names = hb.hyb_trace_summary()
        hb.hyb_trace_enable(False)
        assert list(names) == ["gemm_mfma_256x128.epi%d.n%d.k%d" % (epi, n, k)], (name, names)
        assert err(host(out), ref) < bound, name
        # the first 100 rows alone: 12 tiles, far below one round -> the 128 x 128 kernel; same bits
        small = torch.empty(100, n, device="cuda", dtype=odt)
        kw_s = dict(kw, residual=dev(res[:100])) if kw else {}
        hb.hyb_trace_enable(True)
        hb.hyb_linear(da[:100], dw, db, small, epi, **kw_s)
        torch.cuda.synchronize()
        names = hb.hyb_trace_summary()
        hb.hyb_trace_enable(False)
        assert all(nm.startswith(("gemm_mfma_128x128", "gemm_mfma_64x128")) for nm in names), names
        assert torch.equal(out[:100], small), name
    # in place (out aliases the residual), as the block's fc2 runs
    x = dev(res).clone()
    hb.hyb_linear(da, dw, db, x, hb.HYB_EPI_GATE_RESIDUAL, residual=x, gate=dev(gate), rows_per_gate=1500, gate_stride=n)
    assert err(host(x), res + g_rows * y) < 1e-4
    # several rounds of large tiles (the rows twice: 70 x 13 tiles on 256 CUs): still the large-tile kernel, and each
    # copy of a row gets the bits it got in the single round
    da2 = torch.cat([da, da])
    one, two = torch.empty(m, n, device="cuda", dtype=torch.bfloat16), torch.empty(2 * m, n, device="cuda", dtype=torch.bfloat16)
    hb.hyb_linear(da, dw, db, one, hb.HYB_EPI_GELU_TANH)
    hb.hyb_trace_enable(True)
    hb.hyb_linear(da2, dw, db, two, hb.HYB_EPI_GELU_TANH)
    torch.cuda.synchronize()
    names = hb.hyb_trace_summary()
    hb.hyb_trace_enable(False)
    assert list(names) == ["gemm_mfma_256x128.epi%d.n%d.k%d" % (hb.HYB_EPI_GELU_TANH, n, k)], names
    assert torch.equal(two[:m], one) and torch.equal(two[m:], one)
