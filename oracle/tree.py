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

With a temperature (T > 0) the same tree is filled and verified by sampling.  The paper says nothing here either; what is
used is the published rule that keeps the output exactly the target's: recursive rejection sampling with draws without
replacement (Jeon et al., "Recursive speculative decoding", 2024; for one child per node it is Alg. 3 itself).
  drafting:  the children of a node, in ascending rank, are successive draws from q = softmax(Q_node / T) without
             replacement - the i-th draw by inverse CDF (ascending token index) over q with the earlier draws removed;
  verifying: at the current node with target p = softmax(P_node / T): for each child in rank order with token x,
             accept it with probability min(1, p(x) / q(x)) and move there; on a rejection p <- norm(max(0, p - q)) and
             q <- q with q(x) = 0, renormalised.  When no child is accepted (or the node is a leaf) the emitted token is
             drawn from the current p.
Uniforms: child node v uses position v - 1 (draft stream for its draw, accept stream for its test), the emitted token
position 0 of the residual stream - so a chain-shaped tree consumes exactly the counters of a chain round.
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


def softmax64(logits: np.ndarray, T: float) -> np.ndarray:
    x = logits.astype(np.float64) / T
    e = np.exp(x - x.max())
    return e / e.sum()


def inv_cdf(w: np.ndarray, u: float):
    """Smallest v with sum_{i<=v} w_i > u * sum(w) (ascending index; the last index with weight if rounding leaves none);
    also the distance of u * sum(w) to the nearest CDF step, relative to sum(w)."""
    c = np.cumsum(w)
    Z = c[-1]
    t = float(u) * Z
    v = int(np.searchsorted(c, t, side="right"))
    if v >= len(w):
        v = int(np.nonzero(w > 0)[0][-1])
    lo = c[v - 1] if v > 0 else 0.0
    return v, float(min(abs(c[v] - t), abs(t - lo)) / Z)


def draw_children(logits: np.ndarray, T: float, us) -> tuple:
    """Successive draws without replacement from softmax(logits / T); returns (tokens, margins)."""
    q = softmax64(logits, T)
    toks, mgs = [], []
    for u in us:
        v, mg = inv_cdf(q, u)
        toks.append(v)
        mgs.append(mg)
        q[v] = 0.0
    return toks, mgs


def walk_sampled(P: np.ndarray, Q: np.ndarray, tok, tree: Tree, T: float, u_acc, u_res: float) -> dict:
    """The acceptance walk over a verified tree (see the module docstring).  u_acc[v] = the uniform of child node v.
    Returns path, token and, for the near-tie bookkeeping of lock-step tests, the smallest |u - ratio| met and the margin
    of the final draw."""
    cur, path, gap = 0, [], np.inf
    while True:
        ch = sorted(tree.children(cur), key=lambda j: tree.rank[j])
        p = softmax64(P[cur], T)
        nxt = None
        if ch:
            q = softmax64(Q[cur], T)
            for j in ch:
                x = int(tok[j])
                ratio = p[x] / q[x] if q[x] > 0.0 else np.inf
                gap = min(gap, abs(float(u_acc[j]) - min(1.0, ratio)))
                if float(u_acc[j]) < min(1.0, ratio):
                    nxt = j
                    break
                r = np.maximum(p - q, 0.0)
                Z = r.sum()
                if Z > 0.0:
                    p = r / Z
                q[x] = 0.0
                sq = q.sum()
                if sq > 0.0:
                    q = q / sq
        if nxt is None:
            token, mg = inv_cdf(p, u_res)
            return dict(path=path, token=int(token), gap=float(gap), margin=mg)
        path.append(nxt)
        cur = nxt


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


def tree_round(target, drafter, k: int, st, tree: Tree, tokens=None, outcome=None, T: float = 0.0, seed: int = 0, seq: int = 0) -> dict:
    """One round with a draft tree (greedy for T = 0, sampled otherwise); commits the result.  For lock-step tests:
    tokens = node tokens to use instead of the drafter's own choices (the drafter is run all the same; its own choices are
    returned as own_tok), outcome = (path, token) to commit instead of the walk on this side's logits (returned as
    own_path / own_token all the same)."""
    from . import STREAM_ACCEPT, STREAM_DRAFT, STREAM_RESIDUAL, uniform

    l = st.l
    base = l - 1
    V = target.desc["vocab"]
    tok = np.zeros(tree.n, np.int32)
    tok[0] = st.hist[base]
    own_tok = tok.copy()
    Q = np.zeros((tree.n, V), np.float32)               # drafter logits at the nodes above the deepest level
    draw_margin = np.full(tree.n, np.inf)
    if getattr(drafter, "shares_kv", False):
        st.c[k] = base
    # a drafter head on the target's hidden states: the backlog takes the target's own features, a node below the root the
    # head's estimate at its parent (the reading is stated in oracle/loop.py)
    head = getattr(drafter, "feature_head", False)
    est = np.zeros((tree.n, target.desc["d_model"]), np.float32) if head else None
    for d in range(tree.max_depth):
        nodes = tree.level(d)
        if d == 0 and head:
            c = st.c[k]
            feats = np.zeros((l - c, est.shape[1]), np.float32)
            lo = max(c, 1)
            feats[lo - c:] = st.feat[lo - 1: l - 1]
            Q[0], hid = drafter.forward_hidden(st.hist[c: l], c, "last", feats=feats)
            est[0] = hid[-1]
        elif d == 0:
            Q[0] = drafter.forward(st.hist[st.c[k]: l], st.c[k], "last")          # the committed backlog, ending with the root
        elif head:
            Q[nodes], est[nodes] = drafter.forward_rows_hidden(tok[nodes], [base + i for i in nodes], [base + d] * len(nodes),
                                                               _allow(drafter, tree, base, nodes),
                                                               feats=est[[tree.parent[i] for i in nodes]])
        else:
            Q[nodes] = drafter.forward_rows(tok[nodes], [base + i for i in nodes], [base + d] * len(nodes),
                                            _allow(drafter, tree, base, nodes))
        for i in nodes:
            ch = tree.children(i)
            if ch and T > 0.0:
                ch = sorted(ch, key=lambda j: tree.rank[j])
                drawn, mgs = draw_children(Q[i], T, [uniform(seed, seq, st.t, j - 1, STREAM_DRAFT) for j in ch])
                for j, v, mg in zip(ch, drawn, mgs):
                    own_tok[j] = v
                    draw_margin[j] = mg
                    tok[j] = own_tok[j] if tokens is None else tokens[j]
            elif ch:
                best = ranked_tokens(Q[i], max(tree.rank[j] for j in ch) + 1)
                for j in ch:
                    own_tok[j] = best[tree.rank[j]]
                    tok[j] = own_tok[j] if tokens is None else tokens[j]
    # verify: every node in one pass
    nodes = list(range(tree.n))
    if getattr(st, "feat", None) is not None:
        P, H = target.forward_rows_hidden(tok, [base + i for i in nodes], [base + tree.depth[i] for i in nodes],
                                          _allow(target, tree, base, nodes))
    else:
        P = target.forward_rows(tok, [base + i for i in nodes], [base + tree.depth[i] for i in nodes], _allow(target, tree, base, nodes))
    amax = [int(np.argmax(P[i])) for i in nodes]        # numpy's argmax: first maximum = lowest token on ties
    walk = None
    if T > 0.0:
        # accept: recursive rejection sampling down the tree
        u_acc = np.zeros(tree.n, np.float32)
        for j in range(1, tree.n):
            u_acc[j] = uniform(seed, seq, st.t, j - 1, STREAM_ACCEPT)
        walk = walk_sampled(P, Q, tok, tree, T, u_acc, uniform(seed, seq, st.t, 0, STREAM_RESIDUAL))
        path, token = list(walk["path"]), walk["token"]
    else:
        # accept: follow the target's own greedy choices
        cur, path = 0, []
        while True:
            nxt = [j for j in tree.children(cur) if tok[j] == amax[cur]]
            if not nxt:
                break
            cur = nxt[0]
            path.append(cur)
        token = amax[cur]
    own = (list(path), token)
    if outcome is not None:
        path, token = list(outcome[0]), int(outcome[1])
    n = len(path)
    move_accepted(target, base, path)
    if not getattr(drafter, "shares_kv", False) and not head:
        move_accepted(drafter, base, path[: tree.max_depth - 1])
    st.hist[l: l + n] = tok[path]
    st.hist[l + n] = token
    st.l = l + n + 1
    st.c[k] = st.l - 1 if getattr(drafter, "shares_kv", False) else min(l + n, l + tree.max_depth - 1)
    if getattr(st, "feat", None) is not None:            # the target's features of the committed rows: the root and the accepted nodes
        st.feat[base] = H[0]
        for j, node in enumerate(path):
            st.feat[base + 1 + j] = H[node]
    if head:
        st.c[k] = l                                      # what it computed from estimated features is not kept
    out = dict(k=k, round=st.t, l_before=l, tok=tok, own_tok=own_tok, P=P, Q=Q, amax=amax, path=path, n_acc=n, token=token,
               own_path=own[0], own_token=own[1], walk=walk, draw_margin=draw_margin)
    st.t += 1
    return out


def generate_tree(target, drafters, prompt, n_new: int, tree: Tree, beta: float, policy=None, T: float = 0.0, seed: int = 0) -> dict:
    """MetaSD-UCB generation with tree rounds; reward = N_acc / depth of the tree (Def. 1 with N_max = depth)."""
    from . import SdState, Ucb, reward_be

    prompt = np.asarray(prompt, np.int32)
    l0 = int(prompt.shape[0])
    B = l0 + n_new
    hist = np.zeros(target.max_ctx, np.int32)
    hist[:l0] = prompt
    st = SdState(hist=hist, l=l0, c=[0] * len(drafters))
    if any(getattr(dr, "feature_head", False) for dr in drafters):
        st.feat = np.zeros((target.max_ctx, target.desc["d_model"]), np.float32)
        if l0 > 1:
            _, st.feat[: l0 - 1] = target.forward_hidden(prompt[: l0 - 1], 0, None)
    elif l0 > 1:
        target.forward(prompt[: l0 - 1], 0, None)
    bandit = Ucb(len(drafters), beta)
    rounds = []
    while st.l < B:
        k = bandit.select()
        if policy is not None:
            k = int(policy(st.t))
        r = tree_round(target, drafters[k], k, st, tree, T=T, seed=seed)
        bandit.update(k, reward_be(r["n_acc"], tree.max_depth))
        rounds.append(r)
    return dict(tokens=st.hist[l0:B].copy(), total_len=st.l, rounds=rounds, state=st)
