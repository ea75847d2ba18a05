"""MetaSD-UCB (Alg. 2) of the oracle against a hand-computed run and the classic pull bound."""
import os

import numpy as np

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden", "ucb_alg2_hand.txt")


def test_hand_computed_sequence():
    rows = [ln.split() for ln in open(GOLD) if ln.strip() and not ln.startswith("#")]
    b = oracle.Ucb(3, 1.0)
    for arm, r in enumerate((0.4, 0.6, 0.5)):            # initial sweep in index order
        a, sc = b.select(with_scores=True)
        assert a == arm and np.isnan(sc).all()
        b.update(a, r)
    for t, rew, s0, s1, s2, arm in rows:
        assert b.t == int(t)
        a, sc = b.select(with_scores=True)
        assert np.allclose(sc, [float(s0), float(s1), float(s2)], atol=1e-6)
        assert a == int(arm)
        b.update(a, float(rew))
    assert np.allclose(b.mu, [0.2, 0.4, 0.725]) and b.n.tolist() == [2, 3, 4] and b.t == 9


def test_ties_take_lowest_index_and_beta_scales_bonus():
    b = oracle.Ucb(3, 0.01)
    for a in range(3):
        b.update(b.select(), 0.5)
    a, sc = b.select(with_scores=True)
    assert a == 0 and np.allclose(sc, 0.5 + 0.01 * np.sqrt(2 * np.log(3)))
    one = oracle.Ucb(1, 1.0)
    one.update(one.select(), 1.0)
    assert one.select() == 0                              # K = 1: ln 1 = 0, no bonus, still valid


def test_suboptimal_pulls_respect_ucb1_bound():
    """Theorem 2's proof uses n_i(tau) <= 8 ln(tau)/Delta^2 + 1 + pi^2/3 in expectation (beta = 1)."""
    rng = np.random.default_rng(0)
    means = np.array([0.8, 0.5, 0.3])
    tau, runs = 3000, 20
    pulls = np.zeros(3)
    for _ in range(runs):
        b = oracle.Ucb(3, 1.0)
        for _ in range(tau):
            a = b.select()
            b.update(a, float(rng.random() < means[a]))
        pulls += b.n
    pulls /= runs
    for i in (1, 2):
        delta = means[0] - means[i]
        assert pulls[i] <= 8 * np.log(tau) / delta ** 2 + 1 + np.pi ** 2 / 3
    assert pulls[0] > 0.8 * tau
