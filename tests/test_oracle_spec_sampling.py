"""Pins of the speculative-sampling oracle (Sec. II-A, eqs. ss_accept_prob / ss_residual) to facts it does not
compute itself: a hand-worked example, the theorem that the emitted token follows the target distribution, the
measure of the uniform numbers that lead to each outcome, and the limits in which the rule is greedy
verification or accepts everything."""
import numpy as np
import pytest

from oracle import spec_sampling as ss
from oracle import wisv_oracle as orc


def _dist(rng, n, zeros=0):
    w = rng.gamma(0.7, size=n)
    if zeros:
        w[rng.choice(n, zeros, replace=False)] = 0.0
    return w / w.sum()


def test_hand_worked_example():
    # p_T = (.5 .3 .2 0), p_D = (.2 .5 .1 .2): ratios 2.5, .6, 2, 0 -> alpha = 1, .6, 1, 0;
    # residual weights (.3, 0, .1, 0), total .4
    p_t = np.array([0.5, 0.3, 0.2, 0.0])
    p_d = np.array([0.2, 0.5, 0.1, 0.2])
    assert [ss.accept_prob(p_t, p_d, y) for y in range(4)] == pytest.approx([1.0, 0.6, 1.0, 0.0], abs=1e-15)
    np.testing.assert_allclose(ss.residual(p_t, p_d), [0.3, 0.0, 0.1, 0.0], atol=1e-15)
    r = ss.residual(p_t, p_d)
    assert ss.inverse_cdf(r, 0.0) == 0
    assert ss.inverse_cdf(r, 0.70) == 0        # .28 < .3
    assert ss.inverse_cdf(r, 0.80) == 2        # .32 > .3: token 1 has no weight, token 2 is next
    assert ss.inverse_cdf(r, 0.999) == 2


def test_inverse_cdf_boundaries():
    w = np.array([0.0, 0.25, 0.25, 0.0, 0.5, 0.0])           # dyadic: the sums are exact
    assert ss.inverse_cdf(w, 0.0) == 1                        # leading zero weight is skipped
    assert ss.inverse_cdf(w, 0.25) == 2                       # the inequality is strict: .25 is not > .25
    assert ss.inverse_cdf(w, 0.5) == 4
    assert ss.inverse_cdf(w, np.nextafter(1.0, 0.0)) == 4     # never a trailing zero weight
    assert ss.inverse_cdf(4.0 * w, 0.25) == 2                 # scale free


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_emitted_token_follows_target_distribution(seed):
    # sum over drafted y of p_D(y) [alpha(y) 1{y = x} + (1 - alpha(y)) r(x)] = p_T(x), the property the rule
    # is built for (Sec. II-A); a wrong ratio, a wrong residual or a missing clamp breaks it
    rng = np.random.default_rng(seed)
    n = 7
    p_t, p_d = _dist(rng, n, zeros=seed), _dist(rng, n, zeros=1)
    alpha = np.array([ss.accept_prob(p_t, p_d, y) for y in range(n)])
    r = ss.residual(p_t, p_d)
    assert (r >= 0).all()
    out = p_d * alpha + (p_d * (1.0 - alpha)).sum() * r / r.sum()
    np.testing.assert_allclose(out, p_t, atol=1e-14)


def test_block_outcomes_have_the_right_measure():
    # k = 2: pending token + one drafted token.  Over a fine grid of (u, v) the share of each emitted token,
    # weighted by p_D of the drafted token, is p_T of the position (to the grid's resolution)
    rng = np.random.default_rng(5)
    n, grid = 5, 400
    logits = rng.normal(size=(2, n)) * 1.5
    p_t = np.exp(logits[0] - logits[0].max())
    p_t /= p_t.sum()
    p_d = _dist(rng, n)
    q = np.stack([np.zeros(n), p_d])
    mid = (np.arange(grid) + 0.5) / grid
    emitted = np.zeros(n)
    accepted_share = np.zeros(n)
    for y in range(n):
        for u1 in mid:
            a, tok, _ = ss.verify_block(logits, 3, [3, y], q, [0.5, u1], 0.0)
            if a == 2:                              # accepted: the drafted token stands
                emitted[y] += p_d[y] / grid
                accepted_share[y] += 1.0 / grid
            else:                                   # rejected at 1: the emitted token depends on v only
                assert a == 1
                for v in mid[::8]:
                    _, tok, _ = ss.verify_block(logits, 3, [3, y], q, [0.5, u1], v)
                    emitted[tok] += p_d[y] / grid / len(mid[::8])
    np.testing.assert_allclose(accepted_share, np.minimum(1.0, p_t / p_d), atol=1.5 / grid)
    np.testing.assert_allclose(emitted, p_t, atol=0.03)


def test_pending_token_rule():
    rng = np.random.default_rng(7)
    n, k = 6, 3
    logits, q = rng.normal(size=(k, n)), np.stack([_dist(rng, n) for _ in range(k)])
    a, tok, alpha = ss.verify_block(logits, 4, [2, 1, 0], q, [0.0, 0.0, 0.0], 0.3)
    assert (a, tok, alpha[0]) == (0, 4, 0.0)        # block does not start at the pending token
    a, tok, alpha = ss.verify_block(logits, 2, [2, 1, 0], q, np.full(k, 1.0 - 1e-12), 0.3)
    assert alpha[0] == 1.0 and a >= 1


def test_identical_distributions_accept_everything():
    rng = np.random.default_rng(11)
    n, k = 9, 4
    logits = rng.normal(size=(k, n)) * 2
    q = np.stack([np.zeros(n)] + [ss.softmax(logits[j - 1]) for j in range(1, k)])
    tokens = [5] + list(rng.integers(0, n, k - 1))
    a, tok, alpha = ss.verify_block(logits, 5, tokens, q, np.full(k, np.nextafter(1.0, 0.0)), 0.0)
    assert a == k and (alpha == 1.0).all()
    assert tok == 0                                  # v = 0: the first token with positive probability
    # the bonus token is the inverse CDF of the distribution after the block
    c = np.cumsum(ss.softmax(logits[k - 1]))
    for v in (0.1, 0.5, 0.9):
        assert ss.verify_block(logits, 5, tokens, q, np.zeros(k), v)[1] == int(np.searchsorted(c, v * c[-1], side="right"))


def test_greedy_limit_matches_greedy_verification():
    # one-hot target and drafter distributions: accept iff the drafted token is the target's token, the emitted
    # token is the target's token at the first mismatch -- the greedy rule of Sec. II-A, here taken from the
    # decision code of the round oracle with every gated position rejected
    rng = np.random.default_rng(3)
    n, k = 11, 6
    for trial in range(20):
        t = rng.integers(0, n, k + 1)                       # target tokens of positions 0..k
        draft = t[:k].copy()
        for j in rng.choice(k, rng.integers(0, 3), replace=False):
            draft[j] = (draft[j] + 1 + rng.integers(0, n - 1)) % n
        logits = np.full((k, n), -400.0)
        logits[np.arange(k), t[1:]] = 0.0
        q = np.zeros((k, n))
        q[np.arange(k), draft] = 1.0
        a, tok, _ = ss.verify_block(logits, int(t[0]), draft, q, rng.random(k), rng.random())
        ga, gy, _, _ = orc.decide(draft, t, np.zeros(k, np.int32), np.ones(k, np.float32), 2.0)
        assert (a, tok) == (ga, gy)


def test_nothing_after_the_first_rejection_matters():
    rng = np.random.default_rng(13)
    n, k = 8, 5
    logits = rng.normal(size=(k, n))
    q = np.stack([_dist(rng, n) for _ in range(k)])
    tokens = np.array([1, 2, 3, 4, 5])
    u = np.array([0.0, 0.0, 1.0 - 1e-9, 0.0, 0.0])          # position 2 is rejected unless alpha_2 = 1
    q[2] = 0.0
    q[2, 3] = 1.0                                           # alpha_2 = p_T(3) < 1
    a, tok, _ = ss.verify_block(logits, 1, tokens, q, u, 0.4)
    assert a == 2
    t2, q2, u2, l2 = tokens.copy(), q.copy(), u.copy(), logits.copy()
    t2[3:] = [7, 7]
    q2[3:] = _dist(rng, n)
    u2[3:] = 0.99
    l2[2:] = rng.normal(size=(k - 2, n))                    # rows 2.. only feed positions after the rejected one
    assert ss.verify_block(l2, 1, t2, q2, u2, 0.4)[:2] == (a, tok)
