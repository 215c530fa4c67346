"""Pins of the oracle's reward reduction (Method, Eqs. 2-5 and the group-relative, whitened advantages) against
closed forms, a brute-force double sum and invariances; no GPU."""
import numpy as np
import pytest

import oracle

ACTIONS = [(1, 1, 1, 1, 16), (1, 2, 1, 1, 16), (1, 4, 1, 2, 8), (1, 8, 1, 4, 4)]


def _rand(B, K, T, seed):
    rng = np.random.default_rng(seed)
    return rng.uniform(0.5, 9.0, (B, K, T)), rng.integers(0, len(ACTIONS), (B, K, T)).astype(np.int32)


def test_hinge_is_zero_inside_the_band_and_quadratic_outside():
    assert oracle.hinge_penalty(0.04, 0.05) == 0.0 and oracle.hinge_penalty(-0.05, 0.05) == 0.0
    assert oracle.hinge_penalty(0.15, 0.05) == pytest.approx(0.01)
    assert oracle.hinge_penalty(-0.25, 0.05) == pytest.approx(0.04)


def test_constant_reward_has_the_geometric_closed_form():
    T, gamma, r = 12, 0.85, -2.5
    out = oracle.reward_advantages(np.full((1, 2, T), -r), np.zeros((1, 2, T), np.int32), ACTIONS, [[1, 1, 1]], (1, 1, 1),
                                   0.0, gamma)
    want = [r * (1 - gamma ** (T - t)) / (1 - gamma) for t in range(T)]          # t is 0-based: T - t terms remain
    np.testing.assert_allclose(out["returns"][0, 0], want, rtol=1e-12)


def test_returns_match_the_double_sum_and_suffix_sums_at_gamma_one():
    nll, ids = _rand(2, 3, 9, 1)
    out = oracle.reward_advantages(nll, ids, ACTIONS, [[0.5, 0.5, 0.5]] * 2, (1, 1, 1), 0.05, 0.85)
    for b in range(2):
        for k in range(3):
            for t in range(9):
                brute = sum(0.85 ** (u - t) * -nll[b, k, u] for u in range(t, 9))
                assert out["returns"][b, k, t] == pytest.approx(brute, rel=1e-12)
    out1 = oracle.reward_advantages(nll, ids, ACTIONS, [[0.5, 0.5, 0.5]] * 2, (1, 1, 1), 0.05, 1.0)
    np.testing.assert_allclose(out1["returns"], -np.cumsum(nll[:, :, ::-1], axis=2)[:, :, ::-1], rtol=1e-12)


def test_realised_averages_penalty_and_signal_on_a_hand_example():
    # one input, one schedule of 4 steps: actions 3, 0, 2, 1 -> kappa 1/8, 1, 1/4, 1/2; rho 1/4, 1, 1/2, 1; eta 4/16, 1, 8/16, 1
    ids = np.array([[[3, 0, 2, 1]]], np.int32)
    nll = np.ones((1, 1, 4))
    out = oracle.reward_advantages(nll, ids, ACTIONS, [[0.5, 0.5, 0.9]], (2.0, 3.0, 5.0), 0.05, 0.5)
    np.testing.assert_allclose(out["avg"][0, 0], [0.46875, 0.6875, 0.6875], rtol=1e-15)
    pen = 2.0 * 0.0 + 3.0 * (0.1875 - 0.05) ** 2 + 5.0 * (0.2125 - 0.05) ** 2
    assert out["penalty"][0, 0] == pytest.approx(pen, rel=1e-12)
    np.testing.assert_allclose(out["signal"][0, 0], np.array([-1.875, -1.75, -1.5, -1.0]) - pen, rtol=1e-12)
    # steps 0 and 2 do not count: averages over steps 1 and 3 only
    out = oracle.reward_advantages(nll, ids, ACTIONS, [[0.5, 0.5, 0.9]], (2.0, 3.0, 5.0), 0.05, 0.5, eff=[[0, 1, 0, 1]])
    np.testing.assert_allclose(out["avg"][0, 0], [0.75, 1.0, 1.0], rtol=1e-15)
    # no effective step at all: the averages are the targets and nothing is penalised
    out = oracle.reward_advantages(nll, ids, ACTIONS, [[0.5, 0.5, 0.9]], (2.0, 3.0, 5.0), 0.05, 0.5, eff=[[0, 0, 0, 0]])
    assert out["penalty"][0, 0] == 0.0 and list(out["avg"][0, 0]) == [0.5, 0.5, 0.9]


def test_advantages_are_group_centred_and_whitened():
    nll, ids = _rand(3, 5, 7, 2)
    tg = [[0.6, 0.7, 0.8], [0.3, 0.9, 0.5], [0.9, 0.4, 1.0]]
    out = oracle.reward_advantages(nll, ids, ACTIONS, tg, (4.0, 4.0, 4.0), 0.02, 0.85)
    adv = out["adv"]
    np.testing.assert_allclose(adv.mean(axis=1), 0.0, atol=1e-12)         # over the schedules of an input, at every t
    assert abs(adv.mean()) < 1e-12 and adv.std() == pytest.approx(1.0, abs=1e-6)
    # a per-(input, step) offset common to all schedules and a positive rescaling of every reward change nothing
    off = np.random.default_rng(3).normal(size=(3, 1, 7))
    sig2 = (out["signal"] + off) * 3.0
    c = sig2 - sig2.mean(axis=1, keepdims=True)
    np.testing.assert_allclose((c - c.mean()) / (c.std() + 3e-8), adv, atol=1e-9)
    # the better schedule (lower nll everywhere, same actions) gets the larger advantage at every step
    nll2 = np.stack([np.full((1, 6), 2.0), np.full((1, 6), 3.0)], axis=1)
    out2 = oracle.reward_advantages(nll2, np.zeros((1, 2, 6), np.int32), ACTIONS, [[1, 1, 1]], (1, 1, 1), 0.0, 0.85)
    assert (out2["adv"][0, 0] > out2["adv"][0, 1]).all()
