"""Pins of the oracle's other drafter-selection policies (appendix "Extensions": discounted UCB,
sliding-window UCB, sequential halving / exploration-then-commit, EXP3, uniform random)."""
import math
import os

import numpy as np

import oracle
from oracle import policies as P

GOLD = os.path.join(os.path.dirname(__file__), "golden", "policies_hand.txt")


def gold():
    rows = {}
    for ln in open(GOLD):
        if ln.startswith("#") or not ln.strip():
            continue
        f = ln.split()
        rows.setdefault(f[0], []).append([float(x) for x in f[1:]])
    return rows


def scores(pol):
    return [(pol.mu[i] + pol.beta * math.sqrt(2 * math.log(pol.t) / pol.n[i])) if pol.n[i] else -1.0 for i in range(pol.K)]


def run_hand(pol, rows):
    for a, r in zip(range(3), (0.4, 0.6, 0.5)):
        assert pol.select() == a
        pol.update(a, r)
    for t, r, s0, s1, s2, arm in rows:
        assert pol.t == int(t)
        np.testing.assert_allclose(scores(pol), [s0, s1, s2], atol=2e-6)
        assert pol.select() == int(arm)
        pol.update(int(arm), r)


def test_discounted_ucb_hand_run():
    g = gold()
    pol = P.DiscountedUcb(3, 1.0, 0.5)
    run_hand(pol, g["ducb"])
    np.testing.assert_allclose(pol.mu, g["ducb_final_mu"][0], atol=1e-6)


def test_sliding_window_ucb_hand_run():
    g = gold()
    pol = P.SlidingWindowUcb(3, 1.0, 4)
    run_hand(pol, g["swucb"])
    np.testing.assert_allclose(pol.mu, g["swucb_final_mu"][0], atol=1e-6)
    assert pol.n == [int(x) for x in g["swucb_final_n"][0]]


def test_sequential_halving_hand_run():
    g = gold()
    rew = (0.1, 0.5, 0.3, 0.9, 0.7)
    pol = P.SequentialHalving(5, 15)
    arms = []
    for _ in range(16):
        a = pol.select()
        arms.append(a)
        pol.update(a, rew[a])
    assert arms == [int(x) for x in g["sh_arms"][0]]
    assert pol.alive == [3]


def test_exp3_hand_step_and_invariants():
    g = gold()
    pol = P.Exp3(3, 0.4, seed=5)
    pol.select()
    np.testing.assert_allclose(pol.p, [1 / 3] * 3, rtol=1e-15)
    pol.update(1, 0.9)
    np.testing.assert_allclose(pol.probs(), g["exp3_p_after"][0], atol=1e-6)
    # probabilities always sum to one and never fall below gamma / K; gamma = 1 is uniform
    rng = np.random.default_rng(0)
    for _ in range(2000):
        a = pol.select()
        assert abs(sum(pol.p) - 1.0) < 1e-12 and min(pol.p) >= 0.4 / 3 - 1e-15
        pol.update(a, float(rng.random()))
    assert all(math.isfinite(w) for w in pol.w)          # 2000 rounds: the exact rescale keeps the weights finite
    uni = P.Exp3(4, 1.0, seed=1)
    for _ in range(10):
        a = uni.select()
        uni.update(a, 1.0)
        np.testing.assert_allclose(uni.probs(), [0.25] * 4, rtol=1e-15)


def test_exp3_prefers_the_better_arm_and_random_is_uniform():
    rng = np.random.default_rng(1)
    means = (0.2, 0.8, 0.4)
    pol = P.Exp3(3, 0.4, seed=9)
    for _ in range(3000):
        a = pol.select()
        pol.update(a, float(rng.random() < means[a]))
    assert np.argmax(pol.n) == 1 and pol.n[1] > 0.5 * 3000
    rnd = P.UniformRandom(5, seed=3)
    for _ in range(5000):
        a = rnd.select()
        rnd.update(a, 0.5)
    assert max(abs(c / 5000 - 0.2) for c in rnd.n) < 4 * math.sqrt(0.2 * 0.8 / 5000)


def test_reductions_to_alg2():
    """Discount 1 and a window longer than the run are Alg. 2 exactly."""
    rng = np.random.default_rng(2)
    means = (0.3, 0.6, 0.5, 0.2)
    ucb = oracle.Ucb(4, 0.7)
    d1 = P.DiscountedUcb(4, 0.7, 1.0)
    sw = P.SlidingWindowUcb(4, 0.7, 10**6)
    for _ in range(400):
        a = ucb.select()
        assert d1.select() == a and sw.select() == a
        r = float(rng.random() < means[a])
        ucb.update(a, r); d1.update(a, r); sw.update(a, r)
    np.testing.assert_allclose(d1.mu, ucb.mu, atol=1e-12)
    np.testing.assert_allclose(sw.mu, ucb.mu, atol=1e-12)


def test_nonstationary_policies_follow_a_switch():
    """After the best arm changes, discounted and sliding-window UCB move to the new best arm;
    the stationary index of Alg. 2 with the same beta is slower (the motivation of the appendix)."""
    def run(pol, T=1200):
        rng = np.random.default_rng(4)
        late = 0
        for t in range(T):
            means = (0.8, 0.2) if t < T // 2 else (0.2, 0.8)
            a = pol.select()
            pol.update(a, float(rng.random() < means[a]))
            if t >= T - 200:
                late += a == 1
        return late
    assert run(P.DiscountedUcb(2, 0.3, 0.98)) > 150
    assert run(P.SlidingWindowUcb(2, 0.3, 100)) > 150
    assert run(P.DiscountedUcb(2, 0.3, 0.98)) >= run(oracle.Ucb(2, 0.3))


def test_sequential_halving_keeps_the_best_arm_with_noise():
    wins = 0
    for s in range(40):
        rng = np.random.default_rng(100 + s)
        means = (0.2, 0.35, 0.8, 0.3, 0.25)
        pol = P.SequentialHalving(5, 150)
        for _ in range(200):
            a = pol.select()
            pol.update(a, float(rng.random() < means[a]))
        wins += pol.alive == [2]
    assert wins >= 34
