"""Greedy multi-candidate rounds of the oracle: a tree of draft tokens verified in one target pass with tree
attention (the white-box / multi-draft setting of the paper's Sec. 4, "Number of drafts").

TEST INFRASTRUCTURE ONLY (see the package docstring).

The paper keeps "the original settings with a tree-attention mechanism" of the multi-draft methods and states neither a
tree nor an acceptance rule.  What it does fix is losslessness (paragraph after Alg. 3): in greedy mode the output must
be the target's own greedy continuation.  That determines the rule used here: from the root, follow the child that
carries the target's most likely next token while there is one; the target's most likely token at the last node reached
is emitted.  The tree's shape is an input: node 0 is the root (the last committed token), node i > 0 is the rank[i]-th
most likely next token after node parent[i] according to the drafter (0 = most likely, ties to the lower token), nodes
in breadth-first order.  Node i is held in cache slot l - 1 + i, rotated for position l - 1 + depth(i), and attends to
the committed positions, its ancestors and itself; after acceptance the K/V of the accepted nodes move to the slots of
their positions.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass
class Tree:
    parent: list      # parent[0] = -1
    rank: list        # rank[0] unused

    def __post_init__(self):
        n = len(self.parent)
        assert len(self.rank) == n and n >= 2
        self.n = n
        self.depth = [0] * n
        self.anc = [[0]] + [None] * (n - 1)          # ancestors of a node, the node itself included
        for i in range(1, n):
            p = self.parent[i]
            assert 0 <= p < i
            self.depth[i] = self.depth[p] + 1
            assert self.depth[i] >= self.depth[i - 1], "breadth-first order"
            self.anc[i] = self.anc[p] + [i]
        self.max_depth = self.depth[-1]

    def level(self, d: int) -> list:
        return [i for i in range(self.n) if self.depth[i] == d]

    def children(self, i: int) -> list:
        return [j for j in range(i + 1, self.n) if self.parent[j] == i]

    @staticmethod
    def chain(gamma: int) -> "Tree":
        return Tree([-1] + list(range(gamma)), [0] * (gamma + 1))


def ranked_tokens(logits: np.ndarray, r: int) -> np.ndarray:
    """The r most likely tokens in order, ties to the lower token."""
    return np.argsort(-logits.astype(np.float64), kind="stable")[:r]


def _allow(model, tree: Tree, base: int, nodes: list) -> np.ndarray:
    al = np.zeros((len(nodes), model.max_ctx), np.uint8)
    for r, i in enumerate(nodes):
        al[r, :base] = 1
        al[r, [base + a for a in tree.anc[i]]] = 1
    return al


def move_accepted(model, base: int, path: list):
    """K/V of accepted node path[j] (slot base + path[j]) -> slot of its position base + 1 + j."""
    for which in (0, 1):
        kv = model.kv(which)
        for j, node in enumerate(path):
            kv[:, :, base + 1 + j] = kv[:, :, base + node]


def tree_round(target, drafter, k: int, st, tree: Tree, tokens=None, outcome=None) -> dict:
    """One greedy round with a draft tree; commits the result.  For lock-step tests: tokens = node tokens to use instead
    of the drafter's own choices (the drafter is run all the same; its own choices are returned as own_tok), outcome =
    (path, token) to commit instead of the walk on this side's logits (returned as path / token all the same)."""
    l = st.l
    base = l - 1
    V = target.desc["vocab"]
    tok = np.zeros(tree.n, np.int32)
    tok[0] = st.hist[base]
    own_tok = tok.copy()
    Q = np.zeros((tree.n, V), np.float32)               # drafter logits at the nodes above the deepest level
    if getattr(drafter, "shares_kv", False):
        st.c[k] = base
    for d in range(tree.max_depth):
        nodes = tree.level(d)
        if d == 0:
            Q[0] = drafter.forward(st.hist[st.c[k]: l], st.c[k], "last")          # the committed backlog, ending with the root
        else:
            Q[nodes] = drafter.forward_rows(tok[nodes], [base + i for i in nodes], [base + d] * len(nodes),
                                            _allow(drafter, tree, base, nodes))
        for i in nodes:
            ch = tree.children(i)
            if ch:
                best = ranked_tokens(Q[i], max(tree.rank[j] for j in ch) + 1)
                for j in ch:
                    own_tok[j] = best[tree.rank[j]]
                    tok[j] = own_tok[j] if tokens is None else tokens[j]
    # verify: every node in one pass
    nodes = list(range(tree.n))
    P = target.forward_rows(tok, [base + i for i in nodes], [base + tree.depth[i] for i in nodes], _allow(target, tree, base, nodes))
    # accept: follow the target's own greedy choices
    amax = [int(np.argmax(P[i])) for i in nodes]        # numpy's argmax: first maximum = lowest token on ties
    cur, path = 0, []
    while True:
        nxt = [j for j in tree.children(cur) if tok[j] == amax[cur]]
        if not nxt:
            break
        cur = nxt[0]
        path.append(cur)
    own = (list(path), amax[cur])
    token = amax[cur]
    if outcome is not None:
        path, token = list(outcome[0]), int(outcome[1])
    n = len(path)
    move_accepted(target, base, path)
    if not getattr(drafter, "shares_kv", False):
        move_accepted(drafter, base, path[: tree.max_depth - 1])
    st.hist[l: l + n] = tok[path]
    st.hist[l + n] = token
    st.l = l + n + 1
    st.c[k] = st.l - 1 if getattr(drafter, "shares_kv", False) else min(l + n, l + tree.max_depth - 1)
    out = dict(k=k, round=st.t, l_before=l, tok=tok, own_tok=own_tok, P=P, Q=Q, amax=amax, path=path, n_acc=n, token=token,
               own_path=own[0], own_token=own[1])
    st.t += 1
    return out


def generate_tree(target, drafters, prompt, n_new: int, tree: Tree, beta: float, policy=None) -> dict:
    """Greedy MetaSD-UCB generation with tree rounds; reward = N_acc / depth of the tree (Def. 1 with N_max = depth)."""
    from . import SdState, Ucb, reward_be

    prompt = np.asarray(prompt, np.int32)
    l0 = int(prompt.shape[0])
    B = l0 + n_new
    hist = np.zeros(target.max_ctx, np.int32)
    hist[:l0] = prompt
    st = SdState(hist=hist, l=l0, c=[0] * len(drafters))
    if l0 > 1:
        target.forward(prompt[: l0 - 1], 0, None)
    bandit = Ucb(len(drafters), beta)
    rounds = []
    while st.l < B:
        k = bandit.select()
        if policy is not None:
            k = int(policy(st.t))
        r = tree_round(target, drafters[k], k, st, tree)
        bandit.update(k, reward_be(r["n_acc"], tree.max_depth))
        rounds.append(r)
    return dict(tokens=st.hist[l0:B].copy(), total_len=st.l, rounds=rounds, state=st)
