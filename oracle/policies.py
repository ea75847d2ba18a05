"""Drafter-selection policies other than MetaSD-UCB, as the paper's appendix "Extensions" and its
baselines state them - plain Python, one class per algorithm.

TEST INFRASTRUCTURE ONLY (see the package docstring).  Each class has ``select() -> arm`` and
``update(arm, reward)``; rewards are in [0, 1] (BE or BD).  ``mu``, ``n``, ``t`` mirror what the GPU
library reports through its bandit-state call.

* ``DiscountedUcb``   - Alg. "Discounted UCB in MetaSD": the chosen arm's estimate is its discounted
                        reward sum divided by its pull count; exploration bonus as in Alg. 2.
* ``SlidingWindowUcb``- Alg. "Sliding-window UCB in MetaSD": means and counts over the last tau rounds.
* ``Exp3``            - Alg. "MetaSD-EXP3": exponential weights with uniform mixing gamma.
* ``SequentialHalving`` - Alg. "Sequential Halving" used as the exploration phase of Alg. "Pure
                        exploration-then-commit": after the budget the surviving arm is used for good.
* ``UniformRandom``   - the "Rand" baseline of the main results table.

Readings (the paper is silent or inconsistent here):
  - D-UCB divides by n after counting the current pull (the printed order would divide a sum of
    n+1 terms by n); only the chosen arm's estimate is refreshed, as printed.
  - SW-UCB: an arm with no pull inside the window has no estimate; it is tried first (lowest index).
  - SH: ceil(log2 K) elimination phases, so that one arm is left (with the printed floor two arms of
    five would survive); the better half (largest reward sums) is kept - the printed inequality keeps
    the worse half; ties rank the lower index higher; inside a phase arms are pulled one after the
    other, each n_t = max(1, floor(T / (|S_t| ceil(log2 K)))) times in a row.
  - Random draws (EXP3, Rand): one Philox uniform per round, counter (sequence id, round t, 0,
    stream 3); the arm is the first whose cumulative probability exceeds u.  The sequence id is 0
    for a single sequence; in a batch every sequence has its own bandit drawing under its own id.

Pins: ``tests/test_oracle_policies.py`` (hand-worked runs in ``tests/golden/policies_hand.txt``,
reductions to Alg. 2 for discount 1 / an unbounded window, closed forms of the EXP3 update).
"""
from __future__ import annotations

import math

from . import uniform as _uniform


def _ucb_index(mu, n, t, beta):
    return mu + beta * math.sqrt(2.0 * math.log(t) / n)


def _argmax_first(vals):
    best = 0
    for i in range(1, len(vals)):
        if vals[i] > vals[best]:
            best = i
    return best


class DiscountedUcb:
    def __init__(self, K: int, beta: float, discount: float):
        self.K, self.beta, self.g = K, beta, discount
        self.t = 0
        self.mu = [0.0] * K
        self.n = [0] * K
        self.hist = []                      # (round, arm, reward)

    def select(self) -> int:
        if self.t < self.K:
            return self.t
        return _argmax_first([_ucb_index(self.mu[i], self.n[i], self.t, self.beta) for i in range(self.K)])

    def update(self, arm: int, reward: float):
        self.hist.append((self.t, arm, reward))
        self.n[arm] += 1
        s = 0.0
        for (rs, a, r) in self.hist:        # sum_s gamma^(t-s) r_s [a_s = arm], oldest first
            if a == arm:
                s += self.g ** (self.t - rs) * r
        self.mu[arm] = s / self.n[arm]
        self.t += 1


class SlidingWindowUcb:
    def __init__(self, K: int, beta: float, window: int):
        self.K, self.beta, self.tau = K, beta, window
        self.t = 0
        self.mu = [0.0] * K
        self.n = [0] * K
        self.hist = []                      # (arm, reward) per round

    def select(self) -> int:
        if self.t < self.K:
            return self.t
        for i in range(self.K):
            if self.n[i] == 0:
                return i
        return _argmax_first([_ucb_index(self.mu[i], self.n[i], self.t, self.beta) for i in range(self.K)])

    def update(self, arm: int, reward: float):
        self.hist.append((arm, reward))
        win = self.hist[-self.tau:]
        for i in range(self.K):
            rs = [r for (a, r) in win if a == i]
            self.n[i] = len(rs)
            s = 0.0
            for r in rs:
                s += r
            self.mu[i] = s / len(rs) if rs else 0.0
        self.t += 1


def _draw(probs, u: float) -> int:
    c = 0.0
    for i, p in enumerate(probs):
        c += p
        if c > u:
            return i
    return len(probs) - 1


class Exp3:
    def __init__(self, K: int, gamma: float, seed: int, seq: int = 0):
        self.K, self.g, self.seed, self.seq = K, gamma, seed, seq
        self.t = 0
        self.w = [1.0] * K
        self.p = [1.0 / K] * K
        self.mu = [0.0] * K                 # plain mean reward per arm (reporting only)
        self.n = [0] * K

    def probs(self):
        tot = 0.0
        for w in self.w:
            tot += w
        return [(1.0 - self.g) * (w / tot) + self.g / self.K for w in self.w]

    def select(self) -> int:
        self.p = self.probs()
        return _draw(self.p, float(_uniform(self.seed, self.seq, self.t, 0, 3)))

    def update(self, arm: int, reward: float):
        rhat = reward / self.p[arm]
        self.w[arm] = self.w[arm] * math.exp(self.g * rhat / self.K)
        big = max(self.w)
        if big > 1e100:                     # exact power-of-two rescale: the probabilities do not change
            sc = math.ldexp(1.0, -math.frexp(big)[1])
            self.w = [w * sc for w in self.w]
        self.mu[arm] = (self.mu[arm] * self.n[arm] + reward) / (self.n[arm] + 1)
        self.n[arm] += 1
        self.t += 1


class UniformRandom:
    def __init__(self, K: int, seed: int, seq: int = 0):
        self.K, self.seed, self.seq = K, seed, seq
        self.t = 0
        self.mu = [0.0] * K
        self.n = [0] * K

    def select(self) -> int:
        return _draw([1.0 / self.K] * self.K, float(_uniform(self.seed, self.seq, self.t, 0, 3)))

    def update(self, arm: int, reward: float):
        self.mu[arm] = (self.mu[arm] * self.n[arm] + reward) / (self.n[arm] + 1)
        self.n[arm] += 1
        self.t += 1


class SequentialHalving:
    def __init__(self, K: int, budget: int):
        self.K, self.T = K, budget
        self.t = 0
        self.mu = [0.0] * K
        self.n = [0] * K
        self.alive = list(range(K))
        self.phases = max(1, math.ceil(math.log2(K))) if K > 1 else 0
        self.R = [0.0] * K                  # reward sums of the current phase
        self.pos = 0                        # pulls done in the current phase

    def pulls_per_arm(self) -> int:
        return max(1, self.T // (len(self.alive) * self.phases))

    def select(self) -> int:
        if len(self.alive) == 1:
            return self.alive[0]
        return self.alive[self.pos // self.pulls_per_arm()]

    def update(self, arm: int, reward: float):
        self.mu[arm] = (self.mu[arm] * self.n[arm] + reward) / (self.n[arm] + 1)
        self.n[arm] += 1
        self.t += 1
        if len(self.alive) == 1:
            return
        self.R[arm] += reward
        self.pos += 1
        if self.pos == len(self.alive) * self.pulls_per_arm():
            keep = (len(self.alive) + 1) // 2
            order = sorted(self.alive, key=lambda i: (-self.R[i], i))
            self.alive = sorted(order[:keep])
            self.R = [0.0] * self.K
            self.pos = 0
