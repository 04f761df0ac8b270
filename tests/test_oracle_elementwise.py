"""Pins for the oracle's elementwise functions, normalisations, linear map and embeddings:
torch CPU fp64 library routines, closed forms and pure-Python brute force."""
import math

import numpy as np
import torch
import torch.nn.functional as F

from oracle import hyb_oracle as O


def T(a):
    return torch.from_numpy(np.asarray(a, dtype=np.float64))


def test_silu_gelu_against_library():
    z = np.linspace(-6, 6, 241)
    np.testing.assert_allclose(O.silu(z), F.silu(T(z)).numpy(), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(O.gelu_tanh(z), F.gelu(T(z), approximate="tanh").numpy(), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(O.gelu_erf(z), F.gelu(T(z)).numpy(), rtol=1e-12, atol=1e-15)


def test_gelu_closed_forms():
    assert O.gelu_tanh(0.0) == 0.0 and O.gelu_erf(0.0) == 0.0 and O.silu(0.0) == 0.0
    z = np.linspace(0.1, 5, 50)
    # odd-part identity g(z) - g(-z) = z holds for both forms (tanh and erf are odd)
    np.testing.assert_allclose(O.gelu_tanh(z) - O.gelu_tanh(-z), z, rtol=1e-14)
    np.testing.assert_allclose(O.gelu_erf(z) - O.gelu_erf(-z), z, rtol=1e-14)
    # the two forms differ (a test that would miss swapping them is worthless)
    assert abs(O.gelu_tanh(1.0) - O.gelu_erf(1.0)) > 1e-4
    assert abs(O.gelu_tanh(1.0) - 0.8411919906082768) < 1e-12   # textbook value
    assert abs(O.gelu_erf(1.0) - 0.8413447460685429) < 1e-12    # = Phi(1)
    assert abs(O.silu(1.0) - 1.0 / (1.0 + math.exp(-1.0))) < 1e-15


def test_layer_norm_against_library_and_moments():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((3, 5, 48)) * 3 + 1.5
    y = O.layer_norm(x, 1e-6)
    np.testing.assert_allclose(y, F.layer_norm(T(x), (48,), eps=1e-6).numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(y.mean(-1), 0, atol=1e-13)
    np.testing.assert_allclose(y.var(-1), 1, rtol=1e-5)
    g, b = rng.standard_normal(48), rng.standard_normal(48)
    ya = O.layer_norm_affine(x, g, b, 1e-5)
    np.testing.assert_allclose(ya, F.layer_norm(T(x), (48,), T(g), T(b), eps=1e-5).numpy(), rtol=1e-12, atol=1e-13)
    # eps matters when the variance is tiny: constant row -> exactly zero output
    assert np.all(O.layer_norm(np.full((1, 8), 3.0)) == 0.0)


def test_group_norm_against_library():
    rng = np.random.default_rng(1)
    B, Tn, C = 2, 7, 64
    x = rng.standard_normal((B, Tn, C)) * 2 - 0.7
    g, b = 1 + 0.1 * rng.standard_normal(C), 0.1 * rng.standard_normal(C)
    y = O.group_norm(x, 32, g, b, 1e-5)
    ref = F.group_norm(T(x).permute(0, 2, 1), 32, T(g), T(b), eps=1e-5).permute(0, 2, 1).numpy()
    np.testing.assert_allclose(y, ref, rtol=1e-12, atol=1e-13)
    # brute force for one group: channels 2,3 of sample 1
    vals = [x[1, t, c] for t in range(Tn) for c in (2, 3)]
    mu = sum(vals) / len(vals)
    var = sum((v - mu) ** 2 for v in vals) / len(vals)
    assert abs(y[1, 4, 3] - ((x[1, 4, 3] - mu) / math.sqrt(var + 1e-5) * g[3] + b[3])) < 1e-12


def test_linear_brute_force():
    rng = np.random.default_rng(2)
    x, W, b = rng.standard_normal((3, 5)), rng.standard_normal((4, 5)), rng.standard_normal(4)
    y = O.linear(x, W, b)
    for i in range(3):
        for o in range(4):
            acc = b[o]
            for k in range(5):
                acc += x[i, k] * W[o, k]
            assert abs(y[i, o] - acc) < 1e-13
    np.testing.assert_allclose(O.linear(x, W), F.linear(T(x), T(W)).numpy(), rtol=1e-13)


def test_timestep_embedding_closed_forms():
    e = O.timestep_embedding(np.array([0.0, 0.5]), 256)
    assert e.shape == (2, 256)
    np.testing.assert_array_equal(e[0, :128], 1.0)      # cos(0)
    np.testing.assert_array_equal(e[0, 128:], 0.0)      # sin(0)
    for j in (0, 1, 17, 127):
        f = math.exp(-math.log(10000.0) * j / 128)
        assert abs(e[1, j] - math.cos(500.0 * f)) < 1e-12
        assert abs(e[1, 128 + j] - math.sin(500.0 * f)) < 1e-12
    # j = 0 has frequency 1; the last frequency is 10000^(-127/128)
    assert abs(e[1, 0] - math.cos(500.0)) < 1e-12
    np.testing.assert_allclose(e[1, :128] ** 2 + e[1, 128:] ** 2, 1.0, rtol=1e-14)


def test_timestep_mlp_composition():
    rng = np.random.default_rng(3)
    w1, b1 = rng.standard_normal((8, 256)) * 0.1, rng.standard_normal(8)
    w2, b2 = rng.standard_normal((8, 8)), rng.standard_normal(8)
    t = np.array([0.3])
    e = T(O.timestep_embedding(t, 256))
    ref = F.linear(F.silu(F.linear(e, T(w1), T(b1))), T(w2), T(b2)).numpy()
    np.testing.assert_allclose(O.timestep_mlp(t, w1, b1, w2, b2), ref, rtol=1e-12)


def test_patchify_brute_force_and_inverse():
    rng = np.random.default_rng(4)
    B, Hh, Ww, C, p = 2, 6, 4, 3, 2
    lat = rng.standard_normal((B, Hh, Ww, C))
    tok = O.patchify(lat, p)
    assert tok.shape == (B, (Hh // p) * (Ww // p), p * p * C)
    for b in range(B):
        for py in range(Hh // p):
            for px in range(Ww // p):
                n = py * (Ww // p) + px
                for dy in range(p):
                    for dx in range(p):
                        for c in range(C):
                            assert tok[b, n, (dy * p + dx) * C + c] == lat[b, py * p + dy, px * p + dx, c]
    np.testing.assert_array_equal(O.unpatchify(tok, Hh, Ww, C, p), lat)
