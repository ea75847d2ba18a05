"""Accepted-length statistics of the oracle against the closed forms of the BE-reward lemma
(App. "Proof of Theorem 1": E[N_acc] = (a - a^{N+1})/(1 - a) and the printed variance), the
BE/BD relation (Lemma 2), the expected tokens per round mu^c = (1 - a^{N+1})/(1 - a) of the
single-arm stopping-time lemma, and the numbers the paper prints (tests/golden)."""
import os

import numpy as np
import pytest

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_worked_values.txt")


def golden():
    rows = [ln.split() for ln in open(GOLD) if ln.strip() and not ln.startswith("#")]
    ex = [(float(r[1]), float(r[2])) for r in rows if r[0] == "alpha_nmax2"]
    peak = [float(r[1]) for r in rows if r[0] == "var_be_peak_nmax5"][0]
    return ex, peak


def mean_nacc(a, N):
    return (a - a ** (N + 1)) / (1 - a)


def var_nacc(a, N):
    return a / (1 - a) ** 2 * (1 - (2 * N + 1) * a ** N + (2 * N + 1) * a ** (N + 1) - a ** (2 * N + 1))


def run_constant_alpha(alpha, gamma, N, seed):
    """p = (1, 0), q = (alpha, 1 - alpha): every position has sum min(p, q) = alpha."""
    P = np.array([0.0, -np.inf], np.float32)
    Q = np.log(np.array([alpha, 1 - alpha])).astype(np.float32)
    Qb = np.broadcast_to(Q, (N, gamma, 2))
    Pb = np.broadcast_to(P, (N, gamma + 1, 2))
    d = np.stack([oracle.sample_batch(Qb[:, j], 1.0, oracle.uniform_batch(seed, 0, N, 0, j, 2)) for j in range(gamma)], 1)
    ua = np.stack([oracle.uniform_batch(seed, 0, N, 0, j, 0) for j in range(gamma)], 1)
    return oracle.accept_batch(Pb, Qb, d, 1.0, ua, oracle.uniform_batch(seed, 0, N, 0, 0, 1))


def test_printed_example_nmax2():
    ex, _ = golden()
    N = 400_000
    for alpha, want in ex:
        assert abs(mean_nacc(alpha, 2) - want) < 1e-12           # the closed form reproduces the print
        r = run_constant_alpha(alpha, 2, N, seed=21)
        se = np.sqrt(var_nacc(alpha, 2) / N)
        assert abs(r["n_acc"].mean() - want) < 4.5 * se + 1e-9
        assert np.allclose(r["bd"], alpha, atol=1e-6)             # E[r^BD] = alpha (Lemma on BD statistics)


@pytest.mark.parametrize("alpha", [0.3, 0.6, 0.815, 0.9])
def test_mean_and_variance_nmax5(alpha):
    N, gamma = 400_000, 5
    r = run_constant_alpha(alpha, gamma, N, seed=33)
    n = r["n_acc"].astype(np.float64)
    v = var_nacc(alpha, gamma)
    assert abs(n.mean() - mean_nacc(alpha, gamma)) < 4.5 * np.sqrt(v / N)
    m4 = ((n - n.mean()) ** 4).mean()
    assert abs(n.var() - v) < 4.5 * np.sqrt((m4 - v * v) / N) + 1e-3
    # tokens per round (accepted + one corrected / bonus token)
    assert abs((n + 1).mean() - (1 - alpha ** (gamma + 1)) / (1 - alpha)) < 4.5 * np.sqrt(v / N)
    # BE / BD relation: E[r^BE] = (1 - a^N) / (N (1 - a)) * E[r^BD]
    be = np.mean([oracle.reward_be(int(x), gamma) for x in r["n_acc"][:2000]])
    assert abs(be - n[:2000].mean() / gamma) < 1e-12
    bd = oracle.reward_bd(r["bd"][0])
    assert abs(bd - alpha) < 1e-6
    assert abs(mean_nacc(alpha, gamma) / gamma - (1 - alpha ** gamma) / (gamma * (1 - alpha)) * bd) < 1e-5
    # P(N_acc = n) = a^n (1 - a), P(N_acc = gamma) = a^gamma
    hist = np.bincount(r["n_acc"], minlength=gamma + 1) / N
    want = np.array([alpha ** k * (1 - alpha) for k in range(gamma)] + [alpha ** gamma])
    assert (np.abs(hist - want) < 4.5 * np.sqrt(want * (1 - want) / N) + 1e-9).all()


def test_variance_peak_matches_paper():
    _, peak = golden()
    a = np.linspace(0.5, 0.99, 4901)
    v = var_nacc(a, 5) / 25.0
    assert abs(a[np.argmax(v)] - peak) < 2e-3
