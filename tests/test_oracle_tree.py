"""Pins of the oracle's tree attention and greedy tree rounds (multi-candidate verification, Sec. 4 "Number of drafts").
The paper fixes losslessness (paragraph after Alg. 3); everything here follows from it and from the definition of causal
attention along a root-to-node path."""
import numpy as np
import pytest

import oracle
import workloads as W
from oracle.tree import Tree


@pytest.fixture(scope="module")
def c1():
    cfg = W.config1_tree()
    cfg["tw_np"] = W.to_numpy(cfg["target"][1])
    cfg["dw_np"] = [W.to_numpy(dw) for _, dw in cfg["drafters"]]
    return cfg


def models(cfg, share=False):
    T = oracle.Model(cfg["target"][0], cfg["tw_np"], cfg["max_ctx"])
    D = [oracle.Model(dd, w, cfg["max_ctx"], share_kv_with=T if share else None) for (dd, _), w in zip(cfg["drafters"], cfg["dw_np"])]
    return T, D


def test_chain_shaped_rows_are_the_ordinary_forward(c1):
    """slot = position = pos0 + r with the causal set of visible slots is, by definition, the block forward."""
    A, _ = models(c1)
    B, _ = models(c1)
    prompt = c1["prompt"]
    A.forward(prompt[:9], 0, None)
    B.forward(prompt[:9], 0, None)
    tok = prompt[9:14]
    ref = A.forward(tok, 9, "all")
    allow = np.zeros((5, B.max_ctx), np.uint8)
    for r in range(5):
        allow[r, : 9 + r + 1] = 1
    got = B.forward_rows(tok, 9 + np.arange(5), 9 + np.arange(5), allow)
    assert np.array_equal(ref, got)
    assert np.array_equal(A.kv(0), B.kv(0)) and np.array_equal(A.kv(1), B.kv(1))


def test_every_tree_node_sees_exactly_its_path(c1):
    """Tree attention = causal attention along each root-to-node path: the logits at node i equal the last row of a
    chain forward over (context, tokens on the path to i) in a fresh model - also for siblings, which must not see
    each other, and although node i sits in slot base + i and not in the slot of its position."""
    t = Tree(**W.draft_tree("wide"))
    prompt = c1["prompt"]
    base = 11
    rng = np.random.default_rng(3)
    tok = rng.integers(0, 512, t.n).astype(np.int32)
    tok[0] = prompt[base]
    A, _ = models(c1)
    A.forward(prompt[:base], 0, None)
    allow = np.zeros((t.n, A.max_ctx), np.uint8)
    for i in range(t.n):
        allow[i, :base] = 1
        allow[i, [base + a for a in t.anc[i]]] = 1
    P = A.forward_rows(tok, base + np.arange(t.n), [base + d for d in t.depth], allow)
    for i in range(t.n):
        B, _ = models(c1)
        B.forward(prompt[:base], 0, None)
        ref = B.forward(tok[t.anc[i]], base, "last")
        assert np.array_equal(P[i], ref), i
    # a wrong mask (siblings visible) must change the result: the pin can fail
    allow[2, base + 1] = 1
    P2 = A.forward_rows(tok, base + np.arange(t.n), [base + d for d in t.depth], allow)
    assert not np.array_equal(P2[2], P[2])


@pytest.mark.parametrize("kind", ["wide", "bushy"])
def test_greedy_tree_decoding_is_target_only_greedy_decoding(c1, kind):
    """Losslessness: whatever the drafter and the tree, greedy tree rounds emit the target's own greedy continuation;
    and the caches they leave are those of a model that was simply fed the committed tokens."""
    t = Tree(**W.draft_tree(kind))
    T0, _ = models(c1)
    ref = oracle.ar_decode(T0, c1["prompt"], c1["n_new"], T=0.0)
    for pol, share in ((None, False), (0, False), (2, False), (1, True)):
        T, D = models(c1, share)
        out = oracle.generate_tree(T, D, c1["prompt"], c1["n_new"], t, c1["beta"], policy=None if pol is None else (lambda r, a=pol: a))
        assert np.array_equal(out["tokens"], ref), (pol, share)
        st = out["state"]
        assert st.l - len(c1["prompt"]) == len(out["rounds"]) + sum(r["n_acc"] for r in out["rounds"])
        F, _ = models(c1)
        F.forward(st.hist[: st.l - 1], 0, None)
        for which in (0, 1):
            assert np.array_equal(T.kv(which)[:, :, : st.l - 1], F.kv(which)[:, :, : st.l - 1])
        if pol is not None and not share:                         # the drafter's cache: what it has processed, in position order
            k, ck = pol, st.c[pol]
            Fd = oracle.Model(c1["drafters"][k][0], c1["dw_np"][k], c1["max_ctx"])
            Fd.forward(st.hist[:ck], 0, None)
            assert np.array_equal(D[k].kv(0)[:, :, :ck], Fd.kv(0)[:, :, :ck]) and np.array_equal(D[k].kv(1)[:, :, :ck], Fd.kv(1)[:, :, :ck])
        if pol == 0:                                              # the noiseless drafter: the whole likeliest path, every round
            assert all(r["n_acc"] == t.max_depth for r in out["rounds"])
        if pol is None:                                           # second candidates do get accepted, paths do get deep
            assert any(t.rank[n] > 0 for r in out["rounds"] for n in r["path"]) and max(r["n_acc"] for r in out["rounds"]) >= 3


def test_chain_tree_is_ordinary_greedy_speculation(c1):
    """A chain written as a tree gives the rounds of Alg. 3 in greedy mode: same draft tokens, same accepted lengths."""
    t = Tree(**W.draft_tree("chain5"))
    for arm in (0, 2):
        T, D = models(c1)
        a = oracle.generate(T, D, c1["prompt"], c1["n_new"], 5, 0.0, c1["seed"], c1["beta"], policy=lambda r, a=arm: a)
        T, D = models(c1)
        b = oracle.generate_tree(T, D, c1["prompt"], c1["n_new"], t, c1["beta"], policy=lambda r, a=arm: a)
        assert np.array_equal(a["tokens"], b["tokens"])
        assert [r["n_acc"] for r in a["rounds"]] == [r["n_acc"] for r in b["rounds"]]
        for ra, rb in zip(a["rounds"], b["rounds"]):
            assert np.array_equal(ra["d"], rb["tok"][1:])


def test_a_tree_accepts_at_least_what_its_likeliest_path_accepts(c1):
    """From the same state, a tree that contains the drafter's greedy chain accepts at least as many tokens as that chain."""
    wide, chain = Tree(**W.draft_tree("wide")), Tree(**W.draft_tree("chain5"))
    gains = 0
    for arm in (1, 2):
        for cut in range(5, 17):
            res = []
            for t in (chain, wide):
                T, D = models(c1)
                prompt = c1["prompt"][:cut]
                hist = np.zeros(T.max_ctx, np.int32)
                hist[:cut] = prompt
                T.forward(prompt[:-1], 0, None)
                st = oracle.SdState(hist=hist, l=cut, c=[0] * len(D))
                res.append(oracle.tree_round(T, D[arm], arm, st, t)["n_acc"])
            assert res[1] >= res[0]
            gains += res[1] > res[0]
    assert gains >= 1


# ---------------------------------------------------------------- sampled trees (T > 0)

def test_sampled_chain_tree_is_alg3(c1):
    """One child per node: drawing without replacement is drawing, and recursive rejection sampling is Alg. 3 - with
    the same counters a chain-shaped tree reproduces the chain rounds of the (separately pinned) accept step exactly."""
    t = Tree(**W.draft_tree("chain5"))
    for arm, temp in ((0, 1.0), (2, 0.7)):
        T, D = models(c1)
        a = oracle.generate(T, D, c1["prompt"], c1["n_new"], 5, temp, c1["seed"], c1["beta"], policy=lambda r, a=arm: a)
        T, D = models(c1)
        b = oracle.generate_tree(T, D, c1["prompt"], c1["n_new"], t, c1["beta"], policy=lambda r, a=arm: a, T=temp, seed=c1["seed"])
        assert np.array_equal(a["tokens"], b["tokens"])
        assert [r["n_acc"] for r in a["rounds"]] == [r["n_acc"] for r in b["rounds"]]
        for ra, rb in zip(a["rounds"], b["rounds"]):
            assert np.array_equal(ra["d"], rb["tok"][1:])
        assert max(r["n_acc"] for r in b["rounds"]) >= 2


def _toy_round(rng, tree, ptab, qtab, temp=1.0):
    """One sampled round on a toy in which the target's and the drafter's next-token laws depend on the last token only
    (ptab[x], qtab[x] = logits after token x; the root's token is 0): draws the children, walks, returns the emitted
    tokens of the round in order."""
    from oracle.tree import draw_children, walk_sampled
    tok = np.zeros(tree.n, np.int64)
    for i in range(tree.n):
        ch = sorted(tree.children(i), key=lambda j: tree.rank[j])
        if ch:
            drawn, _ = draw_children(qtab[tok[i]], temp, rng.random(len(ch)))
            for j, v in zip(ch, drawn):
                tok[j] = v
    w = walk_sampled(ptab[tok], qtab[tok], tok, tree, temp, rng.random(tree.n), rng.random())
    return [int(tok[j]) for j in w["path"]] + [w["token"]]


@pytest.mark.parametrize("temp", [1.0, 0.6])
def test_sampled_tree_is_lossless_on_a_toy(temp):
    """Losslessness (the paragraph after Alg. 3), which is all the paper fixes for multi-draft rounds: whatever the
    drafter and the tree, the tokens a round emits are distributed as the target's own sampling.  V = 4, a tree with
    three children at the root and two below the first of them; 200k rounds: the law of the first emitted token is
    p(. | root), and the joint law of the first two (when a second one exists it was either an accepted grandchild or
    the residual / bonus draw after an accepted child) is p(x1 | root) p(x2 | x1) restricted to rounds that emit two -
    compared through the unconditional law of the first token and the conditional law of the second given the first and
    given that the first was an accepted draft (that event depends on x1 only through independent randomness)."""
    rng = np.random.default_rng(11)
    V = 4
    ptab = rng.normal(0, 1.5, (V, V))
    qtab = ptab + rng.normal(0, 1.0, (V, V))
    tree = Tree([-1, 0, 0, 0, 1, 1, 2], [0, 0, 1, 2, 0, 1, 0])
    from oracle.tree import softmax64
    n = 200_000
    first = np.zeros(V)
    second = np.zeros((V, V))
    for _ in range(n):
        out = _toy_round(rng, tree, ptab, qtab, temp)
        first[out[0]] += 1
        if len(out) >= 2:
            second[out[0], out[1]] += 1
    p0 = softmax64(ptab[0], temp)
    sd = np.sqrt(p0 * (1 - p0) / n)
    assert (np.abs(first / n - p0) < 4.5 * sd).all(), (first / n, p0)
    for x in range(V):
        m = second[x].sum()
        if m < 2000:
            continue
        px = softmax64(ptab[x], temp)
        sdx = np.sqrt(px * (1 - px) / m)
        assert (np.abs(second[x] / m - px) < 4.5 * sdx).all(), (x, second[x] / m, px)


def test_sampled_tree_special_cases():
    """q = p: every first child is accepted (ratio 1 > u); disjoint supports: nothing is accepted and the emitted token
    is a draw from p; draws without replacement never repeat a token and follow the renormalised law."""
    from oracle.tree import draw_children, softmax64, walk_sampled
    rng = np.random.default_rng(5)
    V = 16
    tree = Tree(**W.draft_tree("wide"))
    P = rng.normal(0, 2, (tree.n, V)).astype(np.float32)
    tok = rng.integers(0, V, tree.n)
    w = walk_sampled(P, P.copy(), tok, tree, 1.0, rng.random(tree.n) * 0.999, 0.3)
    cur, want = 0, []
    while tree.children(cur):
        cur = min(tree.children(cur), key=lambda j: tree.rank[j])
        want.append(cur)
    assert w["path"] == want
    Pd, Qd = P.copy(), P.copy()
    Pd[:, : V // 2] = -1e9
    Qd[:, V // 2:] = -1e9
    tokq = rng.integers(0, V // 2, tree.n)
    w = walk_sampled(Pd, Qd, tokq, tree, 1.0, rng.random(tree.n), 0.37)
    assert w["path"] == [] and w["token"] >= V // 2
    p = softmax64(Pd[0], 1.0)
    c = np.cumsum(p)
    assert c[w["token"]] > 0.37 >= (c[w["token"] - 1] if w["token"] else 0.0)
    # without replacement: second draw follows q with the first removed
    logits = rng.normal(0, 1, 6)
    q = softmax64(logits, 1.0)
    cnt = np.zeros((6, 6))
    m = 60_000
    for _ in range(m):
        a, b = draw_children(logits, 1.0, rng.random(2))[0]
        assert a != b
        cnt[a, b] += 1
    for a in range(6):
        na = cnt[a].sum()
        want2 = q.copy()
        want2[a] = 0
        want2 /= want2.sum()
        assert abs(na / m - q[a]) < 4.5 * np.sqrt(q[a] * (1 - q[a]) / m)
        assert (np.abs(cnt[a] / na - want2) < 4.5 * np.sqrt(want2 * (1 - want2) / na) + 1e-12).all()


# ---------------------------------------------------------------- drafter heads on the target's hidden states in tree rounds

def _head_models(cfg, eps):
    """Target of config1 with three heads over its first layer; head k weighs the feature input with eps * k (k = 0 ignores it)."""
    T = oracle.Model(cfg["target"][0], cfg["tw_np"], cfg["max_ctx"])
    D = []
    for k in range(3):
        dd, dw, fc = W.feature_head_drafter(cfg["target"][0], cfg["target"][1], 0, eps * k, 300 + k)
        D.append(oracle.Model(dd, W.to_numpy(dw), cfg["max_ctx"], fc=W.to_numpy([fc])[0]))
    return T, D


def test_head_nodes_take_the_estimate_of_their_parent(c1):
    """Every node of a branching tree filled by a head gets the logits of that head run as a chain over the node's own
    root-to-node path in a fresh model - true features for the committed rows, then each step fed the estimate of the
    step before: a node fed a sibling's or an uncle's estimate, or the true feature, fails."""
    t = Tree(**W.draft_tree("wide"))
    prompt = c1["prompt"]
    T, D = _head_models(c1, 0.05)
    hd = D[2]
    l = 12
    hist = np.zeros(T.max_ctx, np.int32)
    hist[:l] = prompt[:l]
    feat = np.zeros((T.max_ctx, T.desc["d_model"]), np.float32)
    _, feat[: l - 1] = T.forward_hidden(prompt[: l - 1], 0, None)
    st = oracle.SdState(hist=hist, l=l, c=[0, 0, 0], feat=feat.copy())
    r = oracle.tree_round(T, hd, 2, st, t)
    tok, Q = r["tok"], r["Q"]
    fin = np.zeros((l, feat.shape[1]), np.float32)
    fin[1:] = feat[: l - 1]
    checked = 0
    for i in range(t.n):
        if not t.children(i):
            continue                                     # logits exist for the nodes that have children
        dd, dw, fc = W.feature_head_drafter(c1["target"][0], c1["target"][1], 0, 0.05 * 2, 302)
        F = oracle.Model(dd, W.to_numpy(dw), c1["max_ctx"], fc=W.to_numpy([fc])[0])
        q, hid = F.forward_hidden(hist[:l], 0, "last", feats=fin)
        for a in t.anc[i][1:]:
            q, hid = F.forward_hidden(tok[a: a + 1], l - 1 + t.depth[a], "last", feats=hid[-1:])
        assert np.array_equal(q, Q[i]), i
        checked += 1
    assert checked >= 5


def test_head_that_ignores_the_features_fills_the_tree_like_the_early_exit_drafter(c1):
    """W_fc = [I | 0]: the head is the target's first layer under the target's norm and head, so its tree rounds are those
    of that early-exit drafter - same node tokens, same paths - although it re-reads the last round's tokens every time."""
    t = Tree(**W.draft_tree("wide"))
    T, D = _head_models(c1, 0.0)
    a = oracle.generate_tree(T, D, c1["prompt"], 40, t, c1["beta"], policy=lambda r: 0)
    dd, dw, _ = W.feature_head_drafter(c1["target"][0], c1["target"][1], 0, 0.0, 300)
    T2 = oracle.Model(c1["target"][0], c1["tw_np"], c1["max_ctx"])
    E = oracle.Model(dd, W.to_numpy(dw), c1["max_ctx"])
    b = oracle.generate_tree(T2, [E], c1["prompt"], 40, t, c1["beta"], policy=lambda r: 0)
    assert np.array_equal(a["tokens"], b["tokens"])
    for ra, rb in zip(a["rounds"], b["rounds"]):
        assert np.array_equal(ra["tok"], rb["tok"]) and ra["path"] == rb["path"]
        assert np.abs(ra["Q"] - rb["Q"]).max() < 1e-5


@pytest.mark.parametrize("temp", [0.0, 1.0])
def test_chain_tree_with_heads_is_the_chain_round_with_heads(c1, temp):
    """A chain written as a tree: the head's estimate passes from node to child exactly as from draft step to draft step."""
    t = Tree(**W.draft_tree("chain5"))
    order = [2, 1, 1, 0, 2]
    T, D = _head_models(c1, 0.05)
    a = oracle.generate(T, D, c1["prompt"], 40, 5, temp, c1["seed"], c1["beta"], policy=lambda r: order[r % 5])
    T, D = _head_models(c1, 0.05)
    b = oracle.generate_tree(T, D, c1["prompt"], 40, t, c1["beta"], policy=lambda r: order[r % 5], T=temp, seed=c1["seed"])
    assert np.array_equal(a["tokens"], b["tokens"])
    for ra, rb in zip(a["rounds"], b["rounds"]):
        assert np.array_equal(ra["d"], rb["tok"][1:]) and ra["n_acc"] == rb["n_acc"]
    assert np.array_equal(a["state"].feat[: a["state"].l - 1], b["state"].feat[: b["state"].l - 1])


def test_greedy_tree_rounds_with_heads_are_lossless_and_keep_the_targets_features(c1):
    t = Tree(**W.draft_tree("wide"))
    T0 = oracle.Model(c1["target"][0], c1["tw_np"], c1["max_ctx"])
    ref = oracle.ar_decode(T0, c1["prompt"], c1["n_new"], T=0.0)
    T, D = _head_models(c1, 0.05)
    order = [0, 2, 1, 1, 2, 0, 0]
    out = oracle.generate_tree(T, D, c1["prompt"], c1["n_new"], t, c1["beta"], policy=lambda r: order[r % len(order)])
    assert np.array_equal(out["tokens"], ref)
    st = out["state"]
    F = oracle.Model(c1["target"][0], c1["tw_np"], c1["max_ctx"])
    _, H = F.forward_hidden(st.hist[: st.l - 1], 0, None)
    assert np.array_equal(st.feat[: st.l - 1], H)
    for which in (0, 1):
        assert np.array_equal(T.kv(which)[:, :, : st.l - 1], F.kv(which)[:, :, : st.l - 1])
    assert sum(r["n_acc"] for r in out["rounds"]) > 0
