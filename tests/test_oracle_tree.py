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
