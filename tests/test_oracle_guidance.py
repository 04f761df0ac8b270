"""Pins for the parts the paper states explicitly: the CFG combine (Sec. 3), the denoising
discrepancy (Eq. 1 and its velocity form), the Euler update of the flow ODE (Sec. 3), the
sigma schedule and the switching rule (Sec. 4.3, Eq. 2-3, Alg. 1)."""
import math
import os

import numpy as np
import pytest

from oracle import hyb_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


# ---------------------------------------------------------------- CFG
def test_cfg_endpoints_and_paper_form():
    v_c, v_u = _rand(0, 2, 50), _rand(1, 2, 50)
    np.testing.assert_allclose(O.cfg_combine(v_c, v_u, 1.0), v_c, rtol=1e-14, atol=1e-15)   # up to one rounding
    np.testing.assert_array_equal(O.cfg_combine(v_c, v_u, 0.0), v_u)
    for w in (0.5, 4.0, 6.0):
        # the paper's eps_c + w (eps_c - eps_u), written out element by element
        ref = np.array([[c + w * (c - u) for c, u in zip(rc, ru)] for rc, ru in zip(v_c, v_u)])
        np.testing.assert_allclose(O.cfg_combine_w(v_c, v_u, w), ref, rtol=1e-15)
        np.testing.assert_allclose(O.cfg_combine(v_c, v_u, 1.0 + w), ref, rtol=1e-13, atol=1e-14)


def test_cfg_linear_in_scale_and_equal_branches():
    v_c, v_u = _rand(2, 40), _rand(3, 40)
    a, b, c = (O.cfg_combine(v_c, v_u, s) for s in (2.0, 5.0, 8.0))
    np.testing.assert_allclose(c - b, b - a, rtol=1e-12, atol=1e-13)
    for s in (0.0, 3.3, 7.0):
        np.testing.assert_array_equal(O.cfg_combine(v_u, v_u, s), v_u)


# ---------------------------------------------------------------- discrepancy
def test_discrepancy_brute_force():
    v_c, v_u = _rand(4, 3, 4, 5), _rand(5, 3, 4, 5)
    d1, d2 = O.branch_discrepancy(v_c, v_u, 1), O.branch_discrepancy(v_c, v_u, 2)
    for b in range(3):
        n1 = n2 = u1 = u2 = 0.0
        for i in range(4):
            for j in range(5):
                diff = v_c[b, i, j] - v_u[b, i, j]
                n1 += abs(diff)
                n2 += diff * diff
                u1 += abs(v_u[b, i, j])
                u2 += v_u[b, i, j] ** 2
        assert abs(d1[b] - n1 / u1) < 1e-14
        assert abs(d2[b] - math.sqrt(n2) / math.sqrt(u2)) < 1e-14


def test_discrepancy_closed_forms():
    v_u = _rand(6, 2, 1000)
    assert np.all(O.branch_discrepancy(v_u, v_u, 1) == 0) and np.all(O.branch_discrepancy(v_u, v_u, 2) == 0)
    for a in (0.25, -0.5, 2.0):
        for p in (1, 2):
            np.testing.assert_allclose(O.branch_discrepancy((1 + a) * v_u, v_u, p), abs(a), rtol=1e-12)
    # invariant under a common scaling of both branches
    v_c = v_u + 0.1 * _rand(7, 2, 1000)
    for p in (1, 2):
        np.testing.assert_allclose(O.branch_discrepancy(3.7 * v_c, 3.7 * v_u, p), O.branch_discrepancy(v_c, v_u, p),
                                   rtol=1e-12)
    # v_u = 1, v_c = 1 + delta e_j: L1 gives delta / n, L2 gives delta / sqrt(n): the norms differ
    n, delta = 400, 0.3
    ones = np.ones((1, n))
    bump = ones.copy()
    bump[0, 17] += delta
    np.testing.assert_allclose(O.branch_discrepancy(bump, ones, 1), delta / n, rtol=1e-12)
    np.testing.assert_allclose(O.branch_discrepancy(bump, ones, 2), delta / math.sqrt(n), rtol=1e-12)
    # not symmetric: the denominator is the unconditional branch
    assert abs(O.branch_discrepancy(2 * ones, ones, 1)[0] - 1.0) < 1e-15
    assert abs(O.branch_discrepancy(ones, 2 * ones, 1)[0] - 0.5) < 1e-15


def test_discrepancy_degenerate_and_per_sample():
    z = np.zeros((1, 8))
    assert O.branch_discrepancy(z, z, 1)[0] == 0.0 and O.branch_discrepancy(z, z, 2)[0] == 0.0
    assert O.branch_discrepancy(z + 1, z, 1)[0] == np.inf and O.branch_discrepancy(z + 1, z, 2)[0] == np.inf
    v_c, v_u = _rand(8, 3, 64), _rand(9, 3, 64)
    full = O.branch_discrepancy(v_c, v_u, 2)
    for b in range(3):     # one ratio per sample, not a ratio of batch sums
        assert full[b] == O.branch_discrepancy(v_c[b:b + 1], v_u[b:b + 1], 2)[0]
    with pytest.raises(ValueError):
        O.branch_discrepancy(v_c, v_u, 3)


# ---------------------------------------------------------------- Euler / schedule
def test_euler_exact_identity_telescoping():
    x, v = _rand(10, 30), _rand(11, 30)
    got = O.euler_step(x, v, 0.5, 0.45)
    for i in range(30):
        assert got[i] == x[i] + (0.45 - 0.5) * v[i]
    np.testing.assert_array_equal(O.euler_step(x, v, 0.3, 0.3), x)
    ts = [1.0, 0.8, 0.55, 0.2, 0.0]
    y = x
    for a, b in zip(ts[:-1], ts[1:]):
        y = O.euler_step(y, v, a, b)
    np.testing.assert_allclose(y, O.euler_step(x, v, 1.0, 0.0), rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(y, x - v, rtol=1e-13, atol=1e-14)        # integrating from t=1 to t=0
    np.testing.assert_array_equal(O.affine_step(x, v, 1.0, -0.05), x + (-0.05) * v)


def test_sigma_schedule():
    s = O.sigma_schedule(28, 3.0)
    assert s.shape == (29,) and s[0] == 1.0 and s[-1] == 0.0
    assert np.all(np.diff(s) < 0)
    np.testing.assert_allclose(O.sigma_schedule(10, 1.0), 1 - np.arange(11) / 10, rtol=1e-15)
    for i in (1, 7, 14, 27):
        u = 1 - i / 28
        assert abs(s[i] - 3 * u / (1 + 2 * u)) < 1e-15
    assert abs(s[14] - 0.75) < 1e-15      # u = 1/2 -> 1.5 / 2


def test_guided_step_composition():
    x, v_c, v_u = _rand(12, 2, 20), _rand(13, 2, 20), _rand(14, 2, 20)
    x_next, v, d1, d2 = O.guided_step(x, v_c, v_u, 7.0, 0.5, 0.45)
    np.testing.assert_allclose(v, v_u + 7.0 * (v_c - v_u), rtol=1e-15)
    np.testing.assert_allclose(x_next, x - 0.05 * v, rtol=1e-13, atol=1e-15)
    np.testing.assert_array_equal(d1, O.branch_discrepancy(v_c, v_u, 1))
    np.testing.assert_array_equal(d2, O.branch_discrepancy(v_c, v_u, 2))


# ---------------------------------------------------------------- switching rule
def _hparams():
    out = {}
    with open(os.path.join(GOLDEN, "switching_hparams.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, L, g, k, cap, T = line.split()
            out[name] = (int(L), float(g), int(k), int(cap), int(T))
    return out


def _u_curve(T, i_min, lo=0.02, hi=0.6):
    """Synthetic U-shaped discrepancy curve: quadratic bowl with its minimum at i_min."""
    i = np.arange(T, dtype=np.float64)
    return lo + (hi - lo) * ((i - i_min) / max(i_min, T - 1 - i_min)) ** 2


def test_switching_rule_on_u_curve_with_paper_hyperparameters():
    hp = _hparams()
    assert hp["SDXL"] == (12, 0.4e-3, 5, 15, 50) and hp["SD3"] == (15, 0.1e-3, 5, 40, 50)
    for name, (L, g, k, cap, T) in hp.items():
        M = _u_curve(T, cap)
        tau1, tau2 = O.switching_points(M, L, g, cap, k)
        assert tau2 == tau1 + k                       # Eq. 3
        assert tau1 <= cap                            # safety cap is an upper bound
        assert 1 <= k < T - tau1
        # brute force: first index i >= L where the mean decline over the window is in [0, g)
        first = next((i for i in range(L, T) if 0 <= (M[i - L] - M[i]) / L < g), None)
        assert tau1 == (cap if first is None else min(first, cap))
        assert [O.stage_of(i, tau1, tau2) for i in (0, tau1, tau1 + 1, tau2 - 1, tau2, T - 1)] == [0, 0, 1, 1, 2, 2]


def test_switching_rule_fires_at_plateau_and_caps():
    # steep fall for 10 steps, then flat: the slope test first holds when the whole window is flat
    M = np.concatenate([np.linspace(1.0, 0.1, 10), np.full(30, 0.1)])
    tau1, tau2 = O.switching_points(M, L=4, g_slope=1e-3, tau_cap=30, k=5)
    assert (tau1, tau2) == (13, 18)                   # M[9] = 0.1 is the first flat value; 9 + L = 13
    assert O.switching_points(M, 4, 1e-3, 11, 5) == (11, 16)        # capped
    # a curve that keeps falling fast never fires: tau1 falls back to the cap
    assert O.switching_points(np.linspace(1.0, 0.0, 40), 4, 1e-3, 20, 7) == (20, 27)
    # a rising window (negative decline) does not fire either
    assert O.switching_points(np.linspace(0.0, 1.0, 40), 4, 1e-3, 9, 2) == (9, 11)


def test_switching_rule_keeps_eq3_bound_on_short_runs():
    """Eq. 3: 1 <= k < T - tau1, so tau2 = tau1 + k is a step of the run.  With the printed SD3 setting
    (L 15, g 1e-4, k 5, tau_cap 40) on a 28-step schedule the cap in force is min(40, 28 - 1 - 5) = 22.
    Expected values are worked by hand from the rule, not computed by the oracle."""
    L, g, k, cap, _ = _hparams()["SD3"]
    T = 28
    # never fires (falls by 1/27 per step, far above g): tau1 = 22, tau2 = 27 = T - 1
    assert O.switching_points(np.linspace(1.0, 0.0, T), L, g, cap, k) == (22, 27)
    # rising curve (negative decline) never fires either
    assert O.switching_points(np.linspace(0.0, 1.0, T), L, g, cap, k) == (22, 27)
    # flat from step 2 on: M[2] = M[17], the window of step 17 = 2 + L is the first flat one
    M = np.concatenate([[1.0, 0.5], np.full(T - 2, 0.1)])
    assert O.switching_points(M, L, g, cap, k) == (17, 22)
    # flat from step 10 on: the test fires at step 25, beyond the cap in force -> (22, 27)
    M = np.concatenate([np.linspace(1.0, 0.2, 10), np.full(T - 10, 0.1)])
    assert O.switching_points(M, L, g, cap, k) == (22, 27)
    # every (tau1, tau2) the rule can return obeys the bound of Eq. 3, whatever the history
    rng = np.random.default_rng(5)
    for T2 in (7, 16, 28, 46, 50):
        for _ in range(50):
            M = np.abs(rng.standard_normal(T2)) * rng.choice([1e-5, 1e-2, 1.0])
            t1, t2 = O.switching_points(M, min(L, T2 - 1), g, cap, k)
            assert 0 <= t1 <= min(cap, T2 - 1 - k) and t2 == t1 + k and 1 <= k < T2 - t1
    # no tau1 >= 0 satisfies k < T - tau1 when k >= T
    with pytest.raises(ValueError):
        O.switching_points(np.ones(5), 2, g, cap, 5)
    # on the 50-step runs of the paper the printed caps are in force unchanged (15 <= 44, 40 <= 44)
    assert O.switching_points(np.linspace(1.0, 0.0, 50), L, g, cap, k) == (40, 45)
