"""Pins for the oracle's accept step (Alg. 3) and its counter-based uniforms.

The closed forms used here are the paper's: a drafted token is accepted with probability
sum_v min(p(v), q(v)) = 1 - d_TV(p, q) (Assumption 1 / Def. 2), and the emitted token is
distributed exactly as the target p (speculative sampling is lossless, Sec. 2.1 and the
paragraph after Alg. 3).  p and q below are computed by numpy in float64, independently of
the oracle's own softmax.
"""
import numpy as np
import pytest

import oracle


def np_softmax(x):
    x = np.asarray(x, np.float64)
    e = np.exp(x - x.max())
    return e / e.sum()


def logits_pair(seed, V=8):
    r = np.random.default_rng(seed)
    P = r.normal(0, 1.5, V).astype(np.float32)
    Q = (P + r.normal(0, 1.0, V)).astype(np.float32)
    return P, Q


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_v8_bruteforce_acceptance_and_marginal(seed):
    """Integrate the oracle over a fine grid of its uniforms for every draft token."""
    V, N = 8, 4000
    P, Q = logits_pair(seed, V)
    p, q = np_softmax(P), np_softmax(Q)
    grid = ((np.arange(N) + 0.5) / N).astype(np.float32)
    Pb = np.broadcast_to(np.stack([P, P]), (N, 2, V))
    Qb = np.broadcast_to(Q[None, None, :], (N, 1, V))
    marginal = np.zeros(V)
    p_accept = 0.0
    for x in range(V):
        d = np.full((N, 1), x, np.int32)
        # (a) accept probability: sweep the accept uniform
        r = oracle.accept_batch(Pb, Qb, d, 1.0, grid[:, None], np.full(N, 0.5, np.float32))
        acc = r["mask"][:, 0].mean()
        assert abs(acc - min(1.0, p[x] / q[x])) <= 1.0 / N + 1e-9
        assert np.allclose(r["ratio"][:, 0], p[x] / q[x], rtol=1e-6)
        assert np.allclose(r["bd"][:, 0], np.minimum(p, q).sum(), rtol=1e-6)
        # (b) residual law: force a rejection (u_acc just below 1 rejects iff p<q), sweep u_res
        res = np.zeros(V)
        if p[x] < q[x] * (1 - 1e-3):
            u_hi = np.full((N, 1), np.float32(1.0 - 2.0 ** -24), np.float32)
            r2 = oracle.accept_batch(Pb, Qb, d, 1.0, u_hi, grid)
            assert (r2["n_acc"] == 0).all()
            res = np.bincount(r2["token"], minlength=V) / N
            want = np.maximum(p - q, 0)
            want /= want.sum()
            assert np.abs(res - want).max() <= 2.0 / N
        marginal[x] += q[x] * acc
        marginal += q[x] * (1 - acc) * res
        p_accept += q[x] * acc
    assert abs(p_accept - np.minimum(p, q).sum()) < 2.0 / N
    assert np.abs(marginal - p).max() < 4.0 / N


def test_identical_distributions_always_accept():
    P, _ = logits_pair(3)
    gamma = 4
    Pm = np.tile(P, (gamma + 1, 1))
    Qm = np.tile(P, (gamma, 1))
    for u in (0.0, 0.3, 1.0 - 2.0 ** -24):
        r = oracle.accept(Pm, Qm, np.arange(gamma) % 8, 1.0, np.full(gamma, u, np.float32), 0.5)
        assert r["n_acc"] == gamma and r["mask"].all()
        assert np.allclose(r["bd"], 1.0)


def test_disjoint_supports_never_accept_and_output_follows_p():
    V, N = 8, 4000
    ninf = np.float32(-np.inf)
    P = np.array([0.3, -0.2, 1.0, 0.1, ninf, ninf, ninf, ninf], np.float32)
    Q = np.array([ninf, ninf, ninf, ninf, 0.0, 0.5, -1.0, 0.2], np.float32)
    p = np_softmax(np.where(np.isfinite(P), P, -1e30))
    grid = ((np.arange(N) + 0.5) / N).astype(np.float32)
    Pb = np.broadcast_to(np.stack([P, P]), (N, 2, V))
    Qb = np.broadcast_to(Q[None, None, :], (N, 1, V))
    for x in (4, 5, 6, 7):
        r = oracle.accept_batch(Pb, Qb, np.full((N, 1), x, np.int32), 1.0,
                                np.zeros((N, 1), np.float32), grid)       # u = 0 still rejects: 0 < 0 is false
        assert (r["n_acc"] == 0).all() and not r["mask"].any()
        assert np.allclose(r["bd"], 0.0)
        hist = np.bincount(r["token"], minlength=V) / N
        assert np.abs(hist - p).max() <= 2.0 / N


def test_strict_inequality_and_first_rejection_index():
    """mask is the raw per-position test; N_acc is the index of the first failure."""
    V, gamma = 8, 4
    P, Q = logits_pair(5, V)
    p, q = np_softmax(P), np_softmax(Q)
    x = int(np.argmin(p / q))                      # a token with ratio < 1
    ratio = p[x] / q[x]
    assert ratio < 0.9
    Pm, Qm = np.tile(P, (gamma + 1, 1)), np.tile(Q, (gamma, 1))
    d = np.full(gamma, x, np.int32)
    u = np.array([ratio * 0.5, ratio * 1.5, ratio * 0.5, ratio * 1.5], np.float32)
    r = oracle.accept(Pm, Qm, d, 1.0, u, 0.25)
    assert r["mask"].tolist() == [1, 0, 1, 0] and r["n_acc"] == 1
    r = oracle.accept(Pm, Qm, d, 1.0, np.full(gamma, ratio * 0.5, np.float32), 0.25)
    assert r["n_acc"] == gamma                      # all accepted: bonus token drawn from p
    N = 2000
    grid = ((np.arange(N) + 0.5) / N).astype(np.float32)
    rb = oracle.accept_batch(np.broadcast_to(Pm, (N, gamma + 1, V)), np.broadcast_to(Qm, (N, gamma, V)),
                             np.broadcast_to(d, (N, gamma)), 1.0,
                             np.full((N, gamma), ratio * 0.5, np.float32), grid)
    assert np.abs(np.bincount(rb["token"], minlength=V) / N - p).max() <= 2.0 / N


def test_temperature_is_applied_to_both_models():
    V = 8
    P, Q = logits_pair(7, V)
    T = 0.7
    p, q = np_softmax(P / T), np_softmax(Q / T)
    r = oracle.accept(np.stack([P, P]), Q[None], [3], T, [0.5], 0.5)
    assert np.isclose(r["ratio"][0], p[3] / q[3], rtol=1e-6)
    assert np.isclose(r["bd"][0], np.minimum(p, q).sum(), rtol=1e-6)
    assert np.allclose(oracle.softmax(P, T), p, rtol=1e-6)


def test_greedy_mode():
    V, gamma = 8, 3
    P = np.array([[0, 5, 1, 0, 0, 0, 0, 0], [2, 2, 0, 0, 0, 0, 0, 0], [0, 0, 0, 0, 0, 0, 9, 0], [1, 0, 0, 0, 0, 0, 0, 7]], np.float32)
    Q = np.zeros((gamma, V), np.float32)
    r = oracle.accept(P, Q, [1, 0, 6], 0.0, np.zeros(gamma, np.float32), 0.9)
    assert r["mask"].tolist() == [1, 1, 1] and r["n_acc"] == 3 and r["token"] == 7   # bonus = argmax of last row
    r = oracle.accept(P, Q, [1, 1, 6], 0.0, np.zeros(gamma, np.float32), 0.9)
    assert r["mask"].tolist() == [1, 0, 1] and r["n_acc"] == 1 and r["token"] == 0   # tie -> lowest index
    assert oracle.sample(P[1], 0.0, 0.99) == 0


def test_inverse_cdf_order_and_margin():
    logits = np.log(np.array([0.1, 0.2, 0.3, 0.4])).astype(np.float32)
    assert [oracle.sample(logits, 1.0, u) for u in (0.0, 0.0999, 0.1001, 0.2999, 0.3001, 0.5999, 0.6001, 0.9999)] \
        == [0, 0, 1, 1, 2, 2, 3, 3]
    t, mg = oracle.sample(logits, 1.0, 0.29, with_margin=True)
    assert t == 1 and abs(mg - 0.01) < 1e-6


def test_two_position_chain_joint_law():
    """The first two emitted tokens follow p1(x1) p2(x2 | x1) when the target's second-position
    distribution depends on the first token (verification rows are conditioned on the drafted prefix)."""
    V, N, seed = 3, 300_000, 11
    r = np.random.default_rng(0)
    P1 = r.normal(0, 1, V).astype(np.float32)
    Q1 = r.normal(0, 1, V).astype(np.float32)
    P2 = r.normal(0, 1, (V, V)).astype(np.float32)      # row = previous token
    Q2 = r.normal(0, 1, (V, V)).astype(np.float32)
    P3 = np.zeros(V, np.float32)
    # round 0, gamma = 2
    d1 = oracle.sample_batch(np.broadcast_to(Q1, (N, V)), 1.0, oracle.uniform_batch(seed, 0, N, 0, 0, 2))
    d2 = oracle.sample_batch(Q2[d1], 1.0, oracle.uniform_batch(seed, 0, N, 0, 1, 2))
    Pb = np.stack([np.broadcast_to(P1, (N, V)), P2[d1], np.broadcast_to(P3, (N, V))], axis=1)
    Qb = np.stack([np.broadcast_to(Q1, (N, V)), Q2[d1]], axis=1)
    ua = np.stack([oracle.uniform_batch(seed, 0, N, 0, j, 0) for j in range(2)], axis=1)
    ur = oracle.uniform_batch(seed, 0, N, 0, 0, 1)
    a = oracle.accept_batch(Pb, Qb, np.stack([d1, d2], 1), 1.0, ua, ur)
    x1 = np.where(a["n_acc"] >= 1, d1, a["token"])
    x2 = np.where(a["n_acc"] == 2, d2, a["token"])      # valid where n_acc >= 1
    # sequences whose first draft was rejected need a second round (gamma = 1) for x2
    idx = np.nonzero(a["n_acc"] == 0)[0]
    e1 = oracle.sample_batch(Q2[x1[idx]], 1.0, oracle.uniform_batch(seed, 0, N, 1, 0, 2)[idx])
    Pb2 = np.stack([P2[x1[idx]], np.broadcast_to(P3, (len(idx), V))], axis=1)
    b = oracle.accept_batch(Pb2, Q2[x1[idx]][:, None, :], e1[:, None], 1.0,
                            oracle.uniform_batch(seed, 0, N, 1, 0, 0)[idx][:, None],
                            oracle.uniform_batch(seed, 0, N, 1, 0, 1)[idx])
    x2[idx] = np.where(b["n_acc"] == 1, e1, b["token"])
    joint = np.zeros((V, V))
    np.add.at(joint, (x1, x2), 1.0)
    joint /= N
    p1 = np_softmax(P1)
    want = np.array([[p1[i] * np_softmax(P2[i])[j] for j in range(V)] for i in range(V)])
    sigma = np.sqrt(want * (1 - want) / N)
    assert (np.abs(joint - want) < 4.5 * sigma).all(), (joint, want)


def test_philox_driven_million_draws():
    V, N, seed = 8, 1_000_000, 1
    P, Q = logits_pair(4, V)
    p, q = np_softmax(P), np_softmax(Q)
    d = oracle.sample_batch(np.broadcast_to(Q, (N, V)), 1.0, oracle.uniform_batch(seed, 0, N, 0, 0, 2))
    assert (np.abs(np.bincount(d, minlength=V) / N - q) < 4.5 * np.sqrt(q * (1 - q) / N)).all()
    r = oracle.accept_batch(np.broadcast_to(np.stack([P, P]), (N, 2, V)), np.broadcast_to(Q, (N, 1, V)),
                            d[:, None], 1.0, oracle.uniform_batch(seed, 0, N, 0, 0, 0)[:, None],
                            oracle.uniform_batch(seed, 0, N, 0, 0, 1))
    alpha = np.minimum(p, q).sum()
    acc = r["mask"][:, 0].mean()
    assert abs(acc - alpha) < 4.5 * np.sqrt(alpha * (1 - alpha) / N)
    out = np.where(r["n_acc"] == 1, d, r["token"])
    hist = np.bincount(out, minlength=V) / N
    assert (np.abs(hist - p) < 4.5 * np.sqrt(p * (1 - p) / N)).all()


def test_philox_structure_and_uniformity():
    """Structural and statistical checks; conformance to the published generator is pinned word for word against
    rocRAND's Philox4x32-10 in tests/test_gpu_philox_pin.py (rocRAND needs a machine with a device)."""
    n = 20000
    outs = np.array([oracle.philox(5, i, 0, 0, 0) for i in range(n)], dtype=np.uint64)
    keys = (outs[:, 0] << np.uint64(32)) | outs[:, 1]
    assert len(np.unique(keys)) == n                       # a bijection never repeats a block
    a = np.array([oracle.philox(5, i, 1, 2, 3) for i in range(2000)], np.uint32)
    b = np.array([oracle.philox(5, i ^ 1, 1, 2, 3) for i in range(2000)], np.uint32)
    flips = np.unpackbits((a ^ b).view(np.uint8)).mean()
    assert 0.49 < flips < 0.51                             # avalanche: one counter bit flips half the output
    c = np.array([oracle.philox(6, i, 1, 2, 3) for i in range(2000)], np.uint32)
    assert 0.49 < np.unpackbits((a ^ c).view(np.uint8)).mean() < 0.51   # key sensitivity
    for word in range(4):
        for pos in (1, 2, 3):                              # every counter word matters
            args = [0, 0, 0, 0]
            args[pos] = 1
            assert (oracle.philox(9, *args) != oracle.philox(9, 0, 0, 0, 0)).any()
    u = oracle.uniform_batch(3, 0, 400_000, 7, 2, 1)
    assert u.min() >= 0.0 and u.max() < 1.0
    assert abs(u.mean() - 0.5) < 4.5 * np.sqrt(1 / 12 / len(u))
    assert abs(u.var() - 1 / 12) < 1e-3
    assert oracle.uniform(3, 5, 7, 2, 1) == u[5]
    assert oracle.uniform(3, 5, 7, 2, 1) != oracle.uniform(3, 5, 7, 2, 0)
