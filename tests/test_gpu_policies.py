"""The library's drafter-selection policies (host code behind metasd_bandit_select / _update) against
the oracle's, arm for arm, through the C ABI; plus one full MetaSD loop driven by a non-UCB policy."""
import numpy as np
import pytest

import oracle
import paper_2604_05417_amd as M
import workloads as W
from oracle import policies as P

pytestmark = pytest.mark.gpu

CASES = [
    ("ucb", 3, dict(), lambda K, seed: oracle.Ucb(K, 0.7)),
    ("ducb", 3, dict(policy_param=0.9), lambda K, seed: P.DiscountedUcb(K, 0.7, 0.9)),
    ("ducb", 5, dict(policy_param=0.5), lambda K, seed: P.DiscountedUcb(K, 0.7, 0.5)),
    ("swucb", 3, dict(policy_window=7), lambda K, seed: P.SlidingWindowUcb(K, 0.7, 7)),
    ("swucb", 5, dict(policy_window=3), lambda K, seed: P.SlidingWindowUcb(K, 0.7, 3)),
    ("exp3", 5, dict(policy_param=0.4), lambda K, seed: P.Exp3(K, 0.4, seed)),
    ("sh", 5, dict(policy_window=60), lambda K, seed: P.SequentialHalving(K, 60)),
    ("sh", 3, dict(policy_window=4), lambda K, seed: P.SequentialHalving(K, 4)),
    ("random", 4, dict(), lambda K, seed: P.UniformRandom(K, seed)),
]


def context(K, policy, **kw):
    cfg = W.config1()
    drafters = (cfg["drafters"] * 2)[:K]
    g = M.MetaSD(cfg["target"], drafters, gamma_max=cfg["gamma"], max_ctx=cfg["max_ctx"], temperature=1.0, seed=11, ucb_beta=0.7,
                 reward="BD", policy=policy, **kw)
    return g, cfg


@pytest.mark.parametrize("case", range(len(CASES)))
def test_policy_matches_oracle_arm_for_arm(case):
    name, K, kw, make = CASES[case]
    g, cfg = context(K, name, **kw)
    ref = make(K, 11)
    rng = np.random.default_rng(100 + case)
    means = rng.random(K)
    for t in range(600):
        if t == 300:
            means = means[::-1].copy()                     # a switch of the best arm half way
        a = g.bandit_select()
        assert a == ref.select(), (name, t)
        r = float(np.clip(means[a] + 0.2 * rng.standard_normal(), 0.0, 1.0))
        g.bandit_update(a, 0, cfg["gamma"], r)
        ref.update(a, r)
        if t % 50 == 49:
            mu, n, tt = g.bandit_state()
            assert tt == ref.t and list(n) == list(ref.n)
            np.testing.assert_allclose(mu, np.asarray(ref.mu, np.float64), rtol=0, atol=1e-12)
    g.set_context(cfg["prompt"])                           # a new query re-initialises the policy
    mu, n, tt = g.bandit_state()
    assert tt == 0 and not n.any()
    assert g.bandit_select() == make(K, 11).select()
    g.close()


@pytest.mark.parametrize("name", ["exp3", "random", "ducb"])
def test_batched_bandits_are_independent(name):
    """Three sequences in one context: each has its own policy state, and the randomised policies draw
    with the sequence's own Philox id (the oracle policy built with seq = b)."""
    cfg = W.config1()
    K = 3
    kw = dict(policy_param=0.4) if name == "exp3" else dict(policy_param=0.8) if name == "ducb" else {}
    g = M.MetaSD(cfg["target"], cfg["drafters"], gamma_max=cfg["gamma"], max_ctx=cfg["max_ctx"], temperature=1.0, seed=11, ucb_beta=0.7,
                 reward="BD", policy=name, batch=3, **kw)
    make = {"exp3": lambda b: P.Exp3(K, 0.4, 11, seq=b), "random": lambda b: P.UniformRandom(K, 11, seq=b),
            "ducb": lambda b: P.DiscountedUcb(K, 0.7, 0.8)}[name]
    refs = [make(b) for b in range(3)]
    rng = np.random.default_rng(5)
    means = rng.random((3, K))
    arms = [[], [], []]
    for t in range(200):
        for b in range(3):
            a = g.bandit_select(seq=b)
            assert a == refs[b].select(), (name, b, t)
            r = float(np.clip(means[b, a] + 0.2 * rng.standard_normal(), 0.0, 1.0))
            g.bandit_update(a, 0, cfg["gamma"], r, seq=b)
            refs[b].update(a, r)
            arms[b].append(a)
    for b in range(3):
        mu, n, tt = g.bandit_state(seq=b)
        assert tt == refs[b].t and list(n) == list(refs[b].n)
        np.testing.assert_allclose(mu, np.asarray(refs[b].mu, np.float64), rtol=0, atol=1e-12)
    assert arms[0] != arms[1] and arms[1] != arms[2]
    g.close()


def test_bad_policy_arguments_are_rejected():
    for kw in (dict(policy="ducb", policy_param=0.0), dict(policy="exp3", policy_param=1.5), dict(policy="swucb", policy_window=0),
               dict(policy="sh", policy_window=0)):
        with pytest.raises(M.MetaSDError) as e:
            context(3, **kw)
        assert e.value.code == -1


def test_full_loop_with_sliding_window_policy():
    """The whole round trip (draft, verify, accept on the GPU) with a non-UCB policy choosing the arm:
    the arm sequence equals the oracle policy fed with the GPU's own rewards, and the loop stays lossless."""
    g, cfg = context(3, "swucb", policy_window=5)
    g.set_context(cfg["prompt"])
    ref = P.SlidingWindowUcb(3, 0.7, 5)
    toks = 0
    while toks < 48:
        k = g.bandit_select()
        assert k == ref.select()
        g.draft(k, cfg["gamma"])
        g.verify(cfg["gamma"])
        n, tok, mask, bd = g.accept(cfg["gamma"])
        g.bandit_update(k, n, cfg["gamma"], bd)
        ref.update(k, bd)
        toks += n + 1
    g.close()
