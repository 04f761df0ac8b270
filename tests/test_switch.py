"""The library's host-side switching controller (Sec. 4.3, Eq. 2-3, Alg. 1) against the oracle's rule.
Runs without a GPU: the controller is host code in libhyb.so."""
import os

import numpy as np
import pytest

from oracle import hyb_oracle as O


@pytest.fixture(scope="module")
def hb():
    from paper_2602_21760_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    binding.lib()
    return binding


def _curves():
    rng = np.random.default_rng(0)
    T = 50
    i = np.arange(T, dtype=np.float64)
    yield 0.02 + 0.58 * ((i - 15) / 34) ** 2                                   # U shape, minimum at 15
    yield 0.02 + 0.58 * ((i - 40) / 40) ** 2                                   # minimum late
    yield np.concatenate([np.linspace(1.0, 0.1, 10), np.full(40, 0.1)])        # fall then plateau
    yield np.linspace(1.0, 0.0, T)                                             # keeps falling: cap
    yield np.linspace(0.0, 1.0, T)                                             # rising: cap
    for _ in range(20):
        yield np.abs(0.3 * np.exp(-i / rng.uniform(3, 20)) + 0.02 + 0.002 * rng.standard_normal(T))


@pytest.mark.parametrize("hp", [(12, 0.4e-3, 15, 5), (15, 0.1e-3, 40, 5), (4, 1e-3, 30, 7), (3, 5e-3, 2, 1)])
def test_controller_matches_oracle_rule(hb, hp):
    L, g, cap, k = hp
    for M in _curves():
        M32 = M.astype(np.float32)
        tau1, tau2 = O.switching_points(M32, L, np.float32(g), cap, k)
        st = hb.hyb_switch_init(len(M), L, g, cap, k)
        stages = [hb.hyb_switch_push(st, float(m)) for m in M32]
        assert (st.tau1, st.tau2) == (tau1, tau2)
        # once the boundaries are known, the reported stages are those of the rule
        for i in range(max(tau1, 0), len(M)):
            assert stages[i] == O.stage_of(i, tau1, tau2)
            assert hb.hyb_switch_stage(st, i) == O.stage_of(i, tau1, tau2)
        assert all(s == 0 for s in stages[:tau1 + 1])                       # warm-up until tau1
        assert tau1 <= cap and tau2 == tau1 + k


def _short_curves(T):
    rng = np.random.default_rng(1)
    i = np.arange(T, dtype=np.float64)
    yield np.linspace(1.0, 0.0, T)                                             # never fires
    yield np.linspace(0.0, 1.0, T)
    yield np.concatenate([[1.0, 0.5], np.full(T - 2, 0.1)])                    # fires as early as the window allows
    yield np.concatenate([np.linspace(1.0, 0.2, 10), np.full(T - 10, 0.1)])    # fires beyond the cap in force
    for _ in range(20):
        yield np.abs(0.3 * np.exp(-i / rng.uniform(2, 12)) + 0.02 + 1e-4 * rng.standard_normal(T))


@pytest.mark.parametrize("T", [28, 21, 50])
def test_controller_on_runs_shorter_than_the_printed_cap(hb, T):
    """The printed SD3 setting (window 15, g 1e-4, k 5, tau_cap 40) on the 28-step schedule of the guided-loop
    workload: the run ends before tau_cap, the cap in force is T - 1 - k (Eq. 3), and the online controller
    arrives at the oracle's (tau1, tau2) with tau2 inside the run."""
    L, g, cap, k = 15, 0.1e-3, 40, 5
    for M in _short_curves(T):
        M32 = M.astype(np.float32)
        tau1, tau2 = O.switching_points(M32, L, np.float32(g), cap, k)
        st = hb.hyb_switch_init(T, L, g, cap, k)
        stages = [hb.hyb_switch_push(st, float(m)) for m in M32]
        assert (st.tau1, st.tau2) == (tau1, tau2)
        assert 0 <= tau1 <= min(cap, T - 1 - k) and tau2 <= T - 1
        assert stages == [O.stage_of(i, tau1, tau2) for i in range(T)]
        assert stages[-1] == 2                                                # the run ends fully connected
    if T == 28:   # hand values: never fired -> (22, 27)
        st = hb.hyb_switch_init(T, L, g, cap, k)
        for m in np.linspace(1.0, 0.0, T):
            hb.hyb_switch_push(st, float(m))
        assert (st.tau1, st.tau2) == (22, 27)


def test_controller_errors(hb):
    with pytest.raises(hb.HybError):
        hb.hyb_switch_init(0, 12, 1e-3, 15, 5)
    with pytest.raises(hb.HybError):
        hb.hyb_switch_init(5000, 12, 1e-3, 15, 5)
    with pytest.raises(hb.HybError):
        hb.hyb_switch_init(5, 2, 1e-3, 15, 5)          # Eq. 3: k < T - tau1 has no solution with k >= T
    st = hb.hyb_switch_init(2, 1, 1e-3, 15, 1)
    hb.hyb_switch_push(st, 0.5)
    hb.hyb_switch_push(st, 0.4)
    with pytest.raises(hb.HybError):
        hb.hyb_switch_push(st, 0.3)
