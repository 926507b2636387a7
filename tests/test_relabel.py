"""The relabelling arithmetic of Sec. V-B (stage 2) against hand-worked numbers and brute force over all action
vectors of small episodes."""
import itertools

import numpy as np
import pytest

from paper_2604_17701_amd import relabel as rl


def test_smoothed_importance_hand_worked():
    # critical mismatches at t = 1 and t = 5, alpha = 1/2: distances (1 0 1 2 1 0 1) -> (.5 1 .5 .25 .5 1 .5)
    bt = rl.smoothed_importance([0, 1, 0, 0, 0, 1, 0], 0.5)
    np.testing.assert_allclose(bt, [0.5, 1.0, 0.5, 0.25, 0.5, 1.0, 0.5])
    assert not rl.smoothed_importance([0, 0, 0], 0.5).any()       # no critical mismatch: nothing to spread
    assert (rl.smoothed_importance([1, 1], 0.3) == 1.0).all()


@pytest.mark.parametrize("seed", range(6))
def test_budget_relabel_is_a_minimiser(seed):
    rng = np.random.default_rng(seed)
    T = int(rng.integers(1, 9))
    b = rng.integers(0, 2, T)
    # any nonnegative weights: the selection rule must be optimal for them, not only for the printed b~
    w = rng.random(T)
    budget = float(rng.integers(0, T + 1)) + 0.5
    a = rl.budget_relabel(b, w, budget)
    assert a.sum() <= budget and (a <= b).all()
    best = min(rl.relabel_objective(b, c, w) for c in itertools.product((0, 1), repeat=T)
               if sum(c) <= budget and all(ci <= bi for ci, bi in zip(c, b)))
    assert rl.relabel_objective(b, a, w) == pytest.approx(best, abs=1e-12)


def test_lagrangian_rule_minimises_the_lagrangian():
    rng = np.random.default_rng(3)
    for _ in range(20):
        T = int(rng.integers(1, 8))
        b, w = rng.integers(0, 2, T), rng.random(T)
        lam, budget = float(rng.random()), 2.0
        a = rl.lagrangian_rule(b, w, lam)
        assert (a <= b).all()
        best = min(rl.lagrangian_value(b, c, w, lam, budget) for c in itertools.product((0, 1), repeat=T)
                   if all(ci <= bi for ci, bi in zip(c, b)))
        assert rl.lagrangian_value(b, a, w, lam, budget) == pytest.approx(best, abs=1e-12)


def test_soft_policy_hand_worked_and_limits():
    b, bt = [1, 0, 1], [1.0, 0.5, 1.0]
    # (1 - 0.4) / 0.2 = 3 -> sigma(3) = 0.9525741268
    np.testing.assert_allclose(rl.soft_policy(b, bt, 0.4, 0.2), [0.9525741268, 0.0, 0.9525741268], atol=1e-9)
    # rho -> 0 recovers the threshold rule; a worse channel (larger lambda) never raises a repair probability
    np.testing.assert_array_equal(np.round(rl.soft_policy(b, bt, 0.4, 1e-6)), rl.lagrangian_rule(b, bt, 0.4))
    assert (rl.soft_policy(b, bt, 0.9, 0.2) <= rl.soft_policy(b, bt, 0.4, 0.2)).all()
    # as printed, every critical mismatch of an episode has b~ = 1: one repair probability per episode
    bt2 = rl.smoothed_importance([0, 1, 0, 1, 1], 0.7)
    pi = rl.soft_policy([0, 1, 0, 1, 1], bt2, 0.6, 0.3)
    assert pi[0] == pi[2] == 0.0 and pi[1] == pi[3] == pi[4]


def test_sampling_and_instances():
    pi = np.array([0.0, 0.25, 1.0])
    np.testing.assert_array_equal(rl.sample_actions(pi, [0.0, 0.25, 0.999]), [0, 0, 1])   # u < pi, strictly
    feats = np.arange(6.0).reshape(3, 2)
    u = np.array([[0.1, 0.1, 0.1], [0.9999, 0.9999, 0.9999]])
    X, y = rl.training_instances(feats, [1, 0, 1], 0.5, [0.2, 0.2], 0.1, u)
    assert X.shape == (6, 2) and (X[:3] == feats).all() and (X[3:] == feats).all()
    np.testing.assert_array_equal(y, [1, 0, 1, 0, 0, 0])        # sigma(8) = 0.99966: 0.1 is below it, 0.9999 is not


def test_bce_hand_worked():
    # -(ln 0.8 + ln 0.5) / 2 = 0.4581453659; with the positive class weighted 3: -(3 ln 0.8 + ln 0.5) / 2
    assert rl.bce_loss([0.8, 0.5], [1, 0]) == pytest.approx(0.4581453659, abs=1e-9)
    assert rl.bce_loss([0.8, 0.5], [1, 0], pos_weight=3.0) == pytest.approx(0.6812889173, abs=1e-9)
