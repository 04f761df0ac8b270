"""Pins for the oracle's attention: brute force, the torch CPU fp64 library routine, and
invariants that hold for softmax attention."""
import math

import numpy as np
import torch
import torch.nn.functional as F

from oracle import hyb_oracle as O


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


def test_softmax_rows_sum_to_one_and_shift_invariant():
    S = _rand(0, 5, 9) * 4
    P = O.softmax_rows(S)
    np.testing.assert_allclose(P.sum(-1), 1.0, rtol=1e-14)
    np.testing.assert_allclose(O.softmax_rows(S + 1000.0), P, rtol=1e-10)
    assert np.all(P > 0)


def test_attention_brute_force_tiny():
    B, H, Nq, Nk, d = 2, 2, 5, 7, 4
    q, k, v = _rand(1, B, H, Nq, d), _rand(2, B, H, Nk, d), _rand(3, B, H, Nk, d)
    o = O.attention(q, k, v)
    assert o.shape == (B, Nq, H * d)
    for b in range(B):
        for h in range(H):
            for i in range(Nq):
                s = [sum(q[b, h, i, c] * k[b, h, j, c] for c in range(d)) / math.sqrt(d) for j in range(Nk)]
                m = max(s)
                e = [math.exp(x - m) for x in s]
                z = sum(e)
                for c in range(d):
                    ref = sum(e[j] / z * v[b, h, j, c] for j in range(Nk))
                    assert abs(o[b, i, h * d + c] - ref) < 1e-13


def test_attention_against_library_sdpa():
    B, H, Nq, Nk, d = 2, 3, 33, 47, 64
    q, k, v = _rand(4, B, H, Nq, d), _rand(5, B, H, Nk, d), _rand(6, B, H, Nk, d)
    ref = F.scaled_dot_product_attention(*(torch.from_numpy(a) for a in (q, k, v)))
    ref = ref.permute(0, 2, 1, 3).reshape(B, Nq, H * d).numpy()
    np.testing.assert_allclose(O.attention(q, k, v), ref, rtol=1e-11, atol=1e-13)
    # explicit scale argument is honoured; non-positive scale means 1/sqrt(d)
    ref2 = F.scaled_dot_product_attention(*(torch.from_numpy(a) for a in (q, k, v)), scale=0.3)
    ref2 = ref2.permute(0, 2, 1, 3).reshape(B, Nq, H * d).numpy()
    np.testing.assert_allclose(O.attention(q, k, v, scale=0.3), ref2, rtol=1e-11, atol=1e-13)
    np.testing.assert_array_equal(O.attention(q, k, v, scale=0.0), O.attention(q, k, v))


def test_attention_with_prescaled_queries_is_the_same_softmax():
    """What the GPU tests of hyb_joint_attention_prescaled compare against: with q' = q * scale * log2(e) the
    weights 2^(q' k) / sum 2^(q' k) are the softmax of q k * scale, i.e. the oracle's attention at scale = ln 2
    on q'; checked here against the library routine on the unscaled q and by brute force in base 2."""
    B, H, Nq, Nk, d = 1, 2, 9, 21, 64
    q, k, v = _rand(14, B, H, Nq, d), _rand(15, B, H, Nk, d), _rand(16, B, H, Nk, d)
    qp = q * (0.125 * math.log2(math.e))
    got = O.attention(qp, k, v, scale=math.log(2.0))
    ref = F.scaled_dot_product_attention(*(torch.from_numpy(a) for a in (q, k, v)))
    np.testing.assert_allclose(got, ref.permute(0, 2, 1, 3).reshape(B, Nq, H * d).numpy(), rtol=1e-11, atol=1e-13)
    for h in range(H):
        for i in range(Nq):
            w = [2.0 ** float(np.dot(qp[0, h, i], k[0, h, j])) for j in range(Nk)]
            row = sum(w[j] * v[0, h, j] for j in range(Nk)) / sum(w)
            np.testing.assert_allclose(got[0, i, h * d:(h + 1) * d], row, rtol=1e-11, atol=1e-13)


def test_attention_invariants():
    B, H, Nq, Nk, d = 1, 2, 6, 10, 8
    q, k, v = _rand(7, B, H, Nq, d), _rand(8, B, H, Nk, d), _rand(9, B, H, Nk, d)
    o = O.attention(q, k, v)
    # all keys equal -> uniform weights -> mean of V
    k_same = np.repeat(k[:, :, :1], Nk, axis=2)
    om = O.attention(q, k_same, v)
    for h in range(H):
        np.testing.assert_allclose(om[0, :, h * d:(h + 1) * d], np.broadcast_to(v[0, h].mean(0), (Nq, d)), rtol=1e-12)
    # one logit far above the rest -> that V row
    k_big = k.copy()
    k_big[0, :, 3] = 200.0 * q[0, :, 2] / np.linalg.norm(q[0, :, 2], axis=-1, keepdims=True)
    ob = O.attention(q, k_big, v)
    for h in range(H):
        np.testing.assert_allclose(ob[0, 2, h * d:(h + 1) * d], v[0, h, 3], atol=1e-9)
    # permuting keys (e.g. text-first instead of image-first concatenation) changes nothing
    perm = np.random.default_rng(10).permutation(Nk)
    np.testing.assert_allclose(O.attention(q, k[:, :, perm], v[:, :, perm]), o, rtol=1e-12)
    # sampled rows and chunked evaluation equal the full computation
    np.testing.assert_array_equal(O.attention(q, k, v, rows=[4, 1]), o[:, [4, 1]])
    np.testing.assert_allclose(O.attention(q, k, v, chunk=4), o, rtol=1e-14)


def test_split_heads_layout():
    y = np.arange(2 * 3 * 8, dtype=np.float64).reshape(2, 3, 8)
    z = O.split_heads(y, 2)
    assert z.shape == (2, 2, 3, 4)
    for b in range(2):
        for n in range(3):
            for h in range(2):
                for i in range(4):
                    assert z[b, h, n, i] == y[b, n, h * 4 + i]
