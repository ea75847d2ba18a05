"""GPU parity of multi-candidate (tree) rounds against the oracle, greedy (T = 0) and sampled (T > 0; the additions for
it are described at TreeLockStep.round).  In greedy mode: the drafter fills a tree of candidates
level by level with tree attention, the target verifies all nodes in one pass, the longest path of the target's own
greedy choices is accepted, the K/V of the accepted nodes move to their positions.  Every round is compared:
  - the children the GPU gave every node are the drafter's most likely tokens by the GPU's own logits (exact);
  - drafter logits at every node above the deepest level and target logits at every node, against the oracle run on
    the GPU's tokens (tolerance);
  - the accepted path and the emitted token are the walk on the GPU's own target logits (exact), and the oracle's own
    outcome (exact for fp32; bf16: differences only where the top-2 gap is inside twice the logit tolerance);
  - committed history, lengths and KV lengths; later rounds run on the compacted caches, so a wrong move shows up as
    a logit mismatch.
For the fp32 configuration the whole output equals the oracle's target-only greedy decoding token for token."""
import numpy as np
import pytest

import oracle
import paper_2604_05417_amd as M
import workloads as W
from lockstep import top2_gap
from oracle.tree import Tree, ranked_tokens
from test_gpu_bf16 import SMALL, TOL, fill_kv, oracle_models

pytestmark = pytest.mark.gpu


class TreeLockStep:
    def __init__(self, gpu, target, drafters, prompt, tree, beta, tol, kv_prefilled=False, temp=0.0, seed=0, feat_prefill=None):
        self.g, self.T, self.D, self.tree, self.tol = gpu, target, drafters, tree, tol
        self.temp, self.seed = temp, seed
        hist = np.zeros(target.max_ctx, np.int32)
        hist[: len(prompt)] = prompt
        self.st = oracle.SdState(hist=hist, l=len(prompt), c=[len(prompt) - 1 if kv_prefilled else 0] * len(drafters))
        if any(getattr(d, "feature_head", False) for d in drafters):     # drafter heads: the target's features are kept too
            self.st.feat = np.zeros((target.max_ctx, target.desc["d_model"]), np.float32)
            if kv_prefilled:                             # synthetic prefix: its features are given like its K/V
                self.st.feat[: len(prompt) - 1] = feat_prefill
            elif len(prompt) > 1:
                _, self.st.feat[: len(prompt) - 1] = target.forward_hidden(prompt[:-1], 0, None)
        elif not kv_prefilled and len(prompt) > 1:
            target.forward(prompt[:-1], 0, None)
        self.bandit = oracle.Ucb(len(drafters), beta)
        self.stats = dict(rounds=0, max_dp=0.0, max_dq=0.0, ties=0, n_acc=[], branch=0)

    def round(self, force_k=None):
        """Sampled rounds (temp > 0) are checked in the same stages, with the sampling rules in place of the greedy ones:
        the children of a node are the oracle's draws without replacement on the GPU's own drafter logits with the same
        uniforms, and the accepted path and emitted token are the oracle's walk (recursive rejection sampling) on the
        GPU's own logits and tokens - exactly, except inside the near-tie windows of the chain protocol (a CDF step
        within 1e-6 of the target, |u - ratio| < 1e-3), which are counted."""
        if self.temp > 0.0:
            return self.round_sampled(force_k)
        g, t, st, tol = self.g, self.tree, self.st, self.tol
        k_gpu, k_or = g.bandit_select(), self.bandit.select()
        assert k_gpu == k_or
        k = k_gpu if force_k is None else force_k
        l = st.l
        g.draft_tree(k, t.parent, t.rank)
        g.verify_tree()
        n, token, path = g.accept_tree()
        Pg = g.peek("P")[: t.n].cpu().numpy()
        Qg = g.peek("Q")[: t.n - 1].cpu().numpy() if t.n - 1 <= g.gamma_max else None
        tok = g.peek("draft")[: t.n].cpu().numpy().copy()
        hist = g.peek("hist")[l: l + n + 1].cpu().numpy()
        inner = [i for i in range(t.n) if t.depth[i] < t.max_depth]
        exact = tol <= 1e-3
        # children by the GPU's own drafter logits
        for i in inner:
            ch = t.children(i)
            if ch:
                best = ranked_tokens(Qg[i], max(t.rank[j] for j in ch) + 1)
                for j in ch:
                    if tok[j] != best[t.rank[j]]:
                        srt = np.sort(Qg[i])[::-1]
                        assert np.min(np.abs(np.diff(srt[: t.rank[j] + 2]))) < 1e-6, f"node {j}: token {tok[j]} is not rank {t.rank[j]} of its parent's logits"
                        self.stats["ties"] += 1
        # the walk on the GPU's own target logits
        amax = [int(np.argmax(Pg[i])) for i in range(t.n)]
        cur, walk = 0, []
        while True:
            nxt = [j for j in t.children(cur) if tok[j] == amax[cur]]
            if not nxt:
                break
            cur = nxt[0]
            walk.append(cur)
        if (walk, amax[cur]) != (path, token):
            assert any(top2_gap(Pg[i]) < 1e-6 for i in [0] + walk), f"round {st.t}: GPU path {path} token {token}, walk on its own logits {walk} {amax[cur]}"
            self.stats["ties"] += 1
        assert (hist[:n] == tok[path]).all() and hist[n] == token
        # the oracle on the GPU's tokens, committing the GPU's outcome
        r = oracle.tree_round(self.T, self.D[k], k, st, t, tokens=tok, outcome=(path, token))
        dq = float(np.abs(r["Q"][inner] - Qg[inner]).max())
        dp = float(np.abs(r["P"] - Pg).max())
        self.stats["max_dq"], self.stats["max_dp"] = max(self.stats["max_dq"], dq), max(self.stats["max_dp"], dp)
        assert dq <= tol and dp <= tol, f"round {st.t - 1}: logits differ by {dq} (drafter) / {dp} (target)"
        same_tokens = np.array_equal(r["own_tok"][1:], tok[1:])        # entry 0 is the root: not a draft token
        if (r["own_path"], r["own_token"]) != (path, token) or not same_tokens:
            tie = any(top2_gap(r["P"][i]) < 2 * tol for i in range(t.n)) or not same_tokens
            assert tie and not exact, (f"round {st.t - 1}: oracle outcome {r['own_path']} {r['own_token']} vs GPU {path} {token}; "
                                       f"oracle tokens {r['own_tok'].tolist()} vs GPU {tok.tolist()}")
            self.stats["ties"] += 1
        self.bandit.update(k, oracle.reward_be(n, t.max_depth))
        g.bandit_update(k, n, t.max_depth)
        lg, kvg, rg = g.state(-1)
        assert (lg, kvg, rg) == (st.l, st.l - 1, st.t)
        assert g.state(k)[1] == st.c[k]
        self.check_features()
        self.stats["rounds"] += 1
        self.stats["n_acc"].append(n)
        self.stats["branch"] += sum(1 for i in path if t.rank[i] > 0)
        return n, token


    def check_features(self):
        """With drafter heads: the table of the target's features holds those of the committed rows (root and accepted nodes
        moved from their slots to their positions)."""
        if self.st.feat is None:
            return
        n = self.st.l - 1
        df = float(np.abs(self.g.peek("feat")[:n].cpu().numpy() - self.st.feat[:n]).max())
        self.stats["max_df"] = max(self.stats.get("max_df", 0.0), df)
        assert df <= self.tol, f"round {self.st.t - 1}: feature table differs by {df}"

    def round_sampled(self, force_k=None):
        from oracle.tree import draw_children, walk_sampled
        g, t, st, tol, T, seed = self.g, self.tree, self.st, self.tol, self.temp, self.seed
        k_gpu, k_or = g.bandit_select(), self.bandit.select()
        assert k_gpu == k_or
        k = k_gpu if force_k is None else force_k
        l, rnd = st.l, st.t
        g.draft_tree(k, t.parent, t.rank)
        g.verify_tree()
        n, token, path = g.accept_tree()
        Pg = g.peek("P")[: t.n].cpu().numpy()
        Qg = np.zeros_like(Pg)
        Qg[: t.n - 1] = g.peek("Q")[: t.n - 1].cpu().numpy()
        tok = g.peek("draft")[: t.n].cpu().numpy().copy()
        tok[0] = st.hist[l - 1]
        hist = g.peek("hist")[l: l + n + 1].cpu().numpy()
        inner = [i for i in range(t.n) if t.depth[i] < t.max_depth]
        # children: the oracle's draws on the GPU's own drafter logits
        for i in inner:
            ch = sorted(t.children(i), key=lambda j: t.rank[j])
            if ch:
                drawn, mgs = draw_children(Qg[i], T, [oracle.uniform(seed, 0, rnd, j - 1, oracle.STREAM_DRAFT) for j in ch])
                for j, v, mg in zip(ch, drawn, mgs):
                    if tok[j] != v:
                        assert mg < 1e-6, f"round {rnd}: node {j}: GPU drew {tok[j]}, the oracle {v} on the same logits (margin {mg})"
                        self.stats["ties"] += 1
                        break                      # later draws of this node start from another urn
        # the walk on the GPU's own logits and tokens
        u_acc = np.zeros(t.n, np.float32)
        for j in range(1, t.n):
            u_acc[j] = oracle.uniform(seed, 0, rnd, j - 1, oracle.STREAM_ACCEPT)
        w = walk_sampled(Pg, Qg, tok, t, T, u_acc, oracle.uniform(seed, 0, rnd, 0, oracle.STREAM_RESIDUAL))
        if (w["path"], w["token"]) != (path, token):
            assert w["gap"] < 1e-3 or w["margin"] < 1e-6, (f"round {rnd}: GPU path {path} token {token}, the oracle's walk on the same logits "
                                                            f"{w['path']} {w['token']} (gap {w['gap']}, margin {w['margin']})")
            self.stats["ties"] += 1
        assert (hist[:n] == tok[path]).all() and hist[n] == token
        # the oracle on the GPU's tokens, committing the GPU's outcome
        r = oracle.tree_round(self.T, self.D[k], k, st, t, tokens=tok, outcome=(path, token), T=T, seed=seed)
        dq = float(np.abs(r["Q"][inner] - Qg[inner]).max())
        dp = float(np.abs(r["P"] - Pg).max())
        self.stats["max_dq"], self.stats["max_dp"] = max(self.stats["max_dq"], dq), max(self.stats["max_dp"], dp)
        assert dq <= tol and dp <= tol, f"round {rnd}: logits differ by {dq} (drafter) / {dp} (target)"
        if tol <= 1e-3 and ((r["own_path"], r["own_token"]) != (path, token) or not np.array_equal(r["own_tok"][1:], tok[1:])):
            # fp32: the oracle's own round is the GPU's, outside the near-tie windows
            assert r["walk"]["gap"] < 1e-3 or r["walk"]["margin"] < 1e-5 or r["draw_margin"].min() < 1e-5, \
                f"round {rnd}: oracle outcome {r['own_path']} {r['own_token']} vs GPU {path} {token}"
            self.stats["ties"] += 1
        self.bandit.update(k, oracle.reward_be(n, t.max_depth))
        g.bandit_update(k, n, t.max_depth)
        lg, kvg, rg = g.state(-1)
        assert (lg, kvg, rg) == (st.l, st.l - 1, st.t)
        assert g.state(k)[1] == st.c[k]
        self.check_features()
        self.stats["rounds"] += 1
        self.stats["n_acc"].append(n)
        self.stats["branch"] += sum(1 for i in path if t.rank[i] > 0)
        return n, token


def make(cfg, tree, tol, share_kv=False, kv_prefilled=False, device="cpu", temp=0.0):
    td, tw = cfg["target"]
    g = M.MetaSD((td, tw), cfg["drafters"], gamma_max=15, max_ctx=cfg["max_ctx"], temperature=temp, seed=cfg["seed"], ucb_beta=cfg["beta"],
                 share_target_kv=share_kv)
    ot, od = oracle_models(cfg, share_kv)
    if kv_prefilled:
        fill_kv(cfg, g, ot, od, len(cfg["prompt"]) - 1, device)
    g.set_context(cfg["prompt"], kv_prefilled=kv_prefilled)
    return g, TreeLockStep(g, ot, od, cfg["prompt"], tree, cfg["beta"], tol, kv_prefilled=kv_prefilled, temp=temp, seed=cfg["seed"])


@pytest.mark.parametrize("kind", ["wide", "bushy", "chain5"])
def test_fp32_tree_rounds_are_lossless(kind):
    """Tiny fp32 configuration (head_dim 32: the plain attention kernel), drafters = the target's layers with noisy heads;
    64 new tokens; the output is the oracle's target-only greedy decoding token for token."""
    cfg = W.config1_tree()
    tree = Tree(**W.draft_tree(kind))
    g, ls = make(cfg, tree, 1e-4)
    l0 = len(cfg["prompt"])
    while ls.st.l < l0 + 64:
        ls.round()
    ref = oracle.ar_decode(oracle.Model(cfg["target"][0], W.to_numpy(cfg["target"][1]), cfg["max_ctx"]), cfg["prompt"], 64, T=0.0)
    assert np.array_equal(ls.st.hist[l0: l0 + 64], ref)
    out = g.peek("hist")[l0: l0 + 64].cpu().numpy()
    assert np.array_equal(out, ref)
    st = ls.stats
    assert st["ties"] == 0 and max(st["n_acc"]) >= 3 and (kind == "chain5" or st["branch"] >= 1), st
    g.close()


@pytest.mark.parametrize("i,share", [(0, False), (2, False), (0, True)])
def test_bf16_tree_rounds(i, share):
    """Small bf16 targets (head_dim 64 and 128: the MFMA attention kernel with the tree mask), prompts spanning several
    attention chunks with a ragged tail, drafters = the target's first layers (all of them, or all but one) with a noisy head,
    with caches of their own or on the target's; arms forced so that a drafter returns after sitting out."""
    s = SMALL[i]
    td = W.model_desc(s["n_layers"], s["d_model"], s["n_heads"], s["n_heads"], s["d_ffn"], s["vocab"], W.SWIGLU, W.BF16)
    tw = W.gen_weights(td, 0)
    drafters = [W.early_exit_drafter(td, tw, e, sg, 300 + k) for k, (e, sg) in enumerate(((s["n_layers"], 0.0), (s["n_layers"], 0.004), (s["n_layers"] - 1, 0.0)))]
    cfg = dict(target=(td, tw), drafters=drafters, prompt=W.prompt_tokens(s["prompt"], s["vocab"], 3), beta=1.0, seed=1, max_ctx=s["prompt"] + 100)
    g, ls = make(cfg, Tree(**W.draft_tree("wide")), TOL, share_kv=share)
    for k in (None, None, None, 1, 0, 1, 2, 0):
        ls.round(k)
    st = ls.stats
    assert st["max_dp"] <= TOL and st["max_dq"] <= TOL and st["ties"] <= 2 and max(st["n_acc"]) >= 3, st
    g.close()


def test_tree_round_with_separate_drafters_and_backlog():
    """Drafters with weights and caches of their own (two layers, narrower than the target): the first pass of a tree
    round consumes the drafter's backlog of committed tokens as a chain, later levels are tree blocks; bushy tree."""
    s = SMALL[0]
    cfg = W.config4(n_layers=s["n_layers"], ctx=s["prompt"], n_new=64, K=2, d_model=s["d_model"], n_heads=s["n_heads"], d_ffn=s["d_ffn"],
                    vocab=s["vocab"], dd_model=s["dd_model"], dn_heads=s["dn_heads"], dd_ffn=s["dd_ffn"])
    cfg["max_ctx"] = s["prompt"] + 100
    g, ls = make(cfg, Tree(**W.draft_tree("bushy")), TOL)
    for k in (None, None, 0, 0, 1, 0):
        ls.round(k)
    st = ls.stats
    assert st["max_dp"] <= TOL and st["max_dq"] <= TOL and st["ties"] <= 2, st
    g.close()


def test_tree_rounds_need_a_single_sequence_context_and_a_valid_tree():
    cfg = W.config1_tree()
    td, tw = cfg["target"]
    t = W.draft_tree("wide")
    g = M.MetaSD((td, tw), cfg["drafters"], gamma_max=15, max_ctx=cfg["max_ctx"], temperature=0.0, seed=1)
    with pytest.raises(M.MetaSDError) as e:                 # no context yet
        g.draft_tree(0, t["parent"], t["rank"])
    assert e.value.code == -3
    g.set_context(cfg["prompt"])
    with pytest.raises(M.MetaSDError):                      # a child before its parent
        g.draft_tree(0, [-1, 2, 0], [0, 0, 0])
    with pytest.raises(M.MetaSDError):                      # not breadth-first
        g.draft_tree(0, [-1, 0, 1, 0], [0, 0, 0, 1])
    with pytest.raises(M.MetaSDError):                      # the same child twice
        g.draft_tree(0, [-1, 0, 0], [0, 1, 1])
    with pytest.raises(M.MetaSDError) as e:                 # verify before draft
        g.verify_tree()
    assert e.value.code == -3
    g.draft_tree(0, t["parent"], t["rank"])
    with pytest.raises(M.MetaSDError) as e:                 # a chain round's verify does not follow a tree draft
        g.verify(5)
    assert e.value.code == -3
    g.verify_tree()
    n, tok, path = g.accept_tree()
    assert 0 <= n <= 5 and len(path) == n
    k = g.bandit_select()
    g.draft(k, 4)                                           # chain rounds and tree rounds mix freely
    g.verify(4)
    g.accept(4)
    g.close()
    g = M.MetaSD((td, tw), cfg["drafters"], gamma_max=5, max_ctx=cfg["max_ctx"], temperature=0.0, seed=1)
    g.set_context(cfg["prompt"])
    with pytest.raises(M.MetaSDError):                      # 13 nodes need gamma_max >= 12
        g.draft_tree(0, t["parent"], t["rank"])
    g.close()


@pytest.mark.parametrize("temp", [0.0, 1.0])
def test_config4_7b_shape_tree_round_full_size(temp):
    """7B-shape target at full size, KV context 2048 (synthetic prefix), separate two-layer drafters: two tree rounds, greedy
    and sampled (13 nodes: a 13-row verification block with the tree mask across 17 attention chunks; vocabulary 32000: draws
    and walk over all eight wavefront segments), every logit compared."""
    cfg = W.config4(device="cuda")
    g, ls = make(cfg, Tree(**W.draft_tree("wide")), TOL, kv_prefilled=True, device="cuda", temp=temp)
    for _ in range(2):
        ls.round()
    st = ls.stats
    assert st["max_dp"] <= TOL and st["max_dq"] <= TOL and st["ties"] <= 1, st
    g.close()


@pytest.mark.parametrize("kind,temp", [("wide", 1.0), ("bushy", 0.7), ("chain5", 1.0)])
def test_fp32_sampled_tree_rounds(kind, temp):
    """Sampled tree rounds on the tiny fp32 configuration: every stage of every round against the oracle (children drawn
    without replacement, the rejection-sampling walk, logits, commits, compacted caches), 64 new tokens; the whole output
    is the oracle's own sampled-tree generation with the same seed token for token (no near-tie on the way); a
    chain-shaped tree gives the tokens of ordinary sampled speculation (the chain loop of the library, same seed)."""
    cfg = W.config1_tree(sigmas=(0.0, 0.05, 0.15))
    tree = Tree(**W.draft_tree(kind))
    g, ls = make(cfg, tree, 1e-4, temp=temp)
    l0 = len(cfg["prompt"])
    while ls.st.l < l0 + 64:
        ls.round(ls.st.t % 3)                      # every arm in turn: the exact drafter accepts everything, the noisy ones branch
    st = ls.stats
    assert st["ties"] == 0 and max(st["n_acc"]) >= 2 and min(st["n_acc"]) < tree.max_depth and (kind == "chain5" or st["branch"] >= 1), st
    tw_np = W.to_numpy(cfg["target"][1])
    T2 = oracle.Model(cfg["target"][0], tw_np, cfg["max_ctx"])
    D2 = [oracle.Model(dd, W.to_numpy(dw), cfg["max_ctx"]) for dd, dw in cfg["drafters"]]
    ref = oracle.generate_tree(T2, D2, cfg["prompt"], 64, tree, cfg["beta"], policy=lambda r: r % 3, T=temp, seed=cfg["seed"])
    out = g.peek("hist")[l0: l0 + 64].cpu().numpy()
    assert np.array_equal(out, ref["tokens"])
    g.close()


def test_bf16_sampled_tree_rounds():
    """Sampled tree rounds on a small bf16 target (head_dim 128: the MFMA attention kernel with the tree mask): the GPU's
    draws and walk are the oracle's on the GPU's own logits, logits within the bf16 tolerance, arms forced so that a
    drafter returns after sitting out."""
    s = SMALL[2]
    td = W.model_desc(s["n_layers"], s["d_model"], s["n_heads"], s["n_heads"], s["d_ffn"], s["vocab"], W.SWIGLU, W.BF16)
    tw = W.gen_weights(td, 0)
    drafters = [W.early_exit_drafter(td, tw, e, sg, 300 + k) for k, (e, sg) in enumerate(((s["n_layers"], 0.0), (s["n_layers"], 0.004), (s["n_layers"] - 1, 0.0)))]
    cfg = dict(target=(td, tw), drafters=drafters, prompt=W.prompt_tokens(s["prompt"], s["vocab"], 3), beta=1.0, seed=1, max_ctx=s["prompt"] + 100)
    g, ls = make(cfg, Tree(**W.draft_tree("wide")), TOL, temp=1.0)
    for k in (None, None, None, 1, 0, 1, 2, 0):
        ls.round(k)
    st = ls.stats
    assert st["ties"] <= 1 and st["rounds"] == 8, st
    g.close()


# ---------------------------------------------------------------- drafter heads on the target's hidden states filling the tree

def make_heads(cfg, tree, tol, temp, eps=0.03, mixed=False):
    """K = 3 heads over the target's first layer (feature weight eps * (k + 1)); mixed: drafter 1 stays an ordinary drafter."""
    td, tw = cfg["target"]
    tw_np = W.to_numpy(tw)
    cache = {id(t): a for t, a in zip(tw, tw_np)}
    drafters, heads, od = [], {}, []
    for k in range(3):
        if mixed and k == 1:
            dd, dw = cfg["drafters"][1]
            fc = None
        else:
            dd, dw, fc = W.feature_head_drafter(td, tw, 0, eps * (k + 1), 300 + k)
            heads[k] = fc
        drafters.append((dd, dw))
        arrs = [cache[id(t)] if id(t) in cache else W.to_numpy([t])[0] for t in dw]
        od.append(oracle.Model(dd, arrs, cfg["max_ctx"], fc=None if fc is None else W.to_numpy([fc])[0]))
    g = M.MetaSD((td, tw), drafters, gamma_max=15, max_ctx=cfg["max_ctx"], temperature=temp, seed=cfg["seed"], ucb_beta=cfg["beta"], heads=heads)
    g.set_context(cfg["prompt"])
    return g, TreeLockStep(g, oracle.Model(td, tw_np, cfg["max_ctx"]), od, cfg["prompt"], tree, cfg["beta"], tol, temp=temp, seed=cfg["seed"])


@pytest.mark.parametrize("temp", [0.0, 1.0])
@pytest.mark.parametrize("kind,mixed", [("wide", False), ("bushy", True)])
def test_config1_tree_rounds_with_drafter_heads(kind, mixed, temp):
    """fp32: heads fill the tree (every node takes the head's estimate at its parent), the target's features of the root and
    of the accepted nodes end up at their positions; 48 new tokens in lock-step, greedy: the target's own greedy continuation."""
    cfg = W.config1_tree()
    tree = Tree(**W.draft_tree(kind))
    g, ls = make_heads(cfg, tree, 1e-4, temp, mixed=mixed)
    order = [0, 2, 1, 1, 2, 0, 0]
    B = len(cfg["prompt"]) + 48
    while ls.st.l < B:
        ls.round(order[ls.st.t % len(order)])
    st = ls.stats
    assert st["ties"] <= 1 and st["max_dp"] <= 1e-4 and st["max_dq"] <= 1e-4 and st["max_df"] <= 1e-4, st
    if temp == 0.0:
        ref = oracle.ar_decode(oracle.Model(cfg["target"][0], W.to_numpy(cfg["target"][1]), cfg["max_ctx"]), cfg["prompt"], 48, T=0.0)
        assert np.array_equal(ls.st.hist[len(cfg["prompt"]): B], ref)
    g.close()


@pytest.mark.parametrize("temp", [0.0, 1.0])
def test_small_bf16_tree_rounds_with_drafter_heads(temp):
    """bf16 (head_dim 64, MFMA path, the 13-row verification block through the residual kernels with the features kept)."""
    cfg = W.config4(n_layers=2, ctx=45, n_new=64, K=2, d_model=256, n_heads=4, d_ffn=736, vocab=1040, dd_model=128, dn_heads=2, dd_ffn=160)
    cfg["max_ctx"] = 45 + 100
    tree = Tree(**W.draft_tree("wide"))
    g, ls = make_heads(cfg, tree, TOL, temp, eps=0.02, mixed=True)
    order = [0, 1, 2, 2, 0]
    for _ in range(8):
        ls.round(order[ls.st.t % len(order)])
    assert ls.stats["max_dp"] <= TOL and ls.stats["max_dq"] <= TOL and ls.stats["max_df"] <= TOL, ls.stats
    g.close()


@pytest.mark.parametrize("temp", [0.0, 1.0])
def test_config4_7b_shape_tree_rounds_with_drafter_heads(temp):
    """The 7B shape at full size: two one-layer heads (W_fc [4096, 8192]) fill the 13-node tree, synthetic K/V and feature
    prefix of 2047 positions on both sides; one round per head and a return to the first."""
    import torch
    cfg = W.config4(device="cuda", K=1)
    td, tw = cfg["target"]
    n0 = len(cfg["prompt"]) - 1
    tw_np = W.to_numpy(tw)
    cache = {id(t): a for t, a in zip(tw, tw_np)}
    drafters, heads, od = [], {}, []
    for k in range(2):
        dd, dw, fc = W.feature_head_drafter(td, tw, k, 0.01 * (k + 1), 300 + k)
        drafters.append((dd, dw))
        heads[k] = fc
        od.append(oracle.Model(dd, [cache[id(t)] for t in dw], cfg["max_ctx"], fc=W.to_numpy([fc])[0]))
    ot = oracle.Model(td, tw_np, cfg["max_ctx"])
    g = M.MetaSD((td, tw), drafters, gamma_max=15, max_ctx=cfg["max_ctx"], temperature=temp, seed=cfg["seed"], ucb_beta=cfg["beta"], heads=heads)
    for i, (desc, kv_gpu, om) in enumerate([(td, g.kv_target, ot)] + [(dd, g.kv_drafters[k], od[k]) for k, (dd, _) in enumerate(drafters)]):
        kk, vv = W.kv_fill(desc, n0, cfg["kv_seed"] + i, device="cuda")
        kv_gpu[:, 0, :, :n0] = kk
        kv_gpu[:, 1, :, :n0] = vv
        om.kv(0)[:, :, :n0] = kk.float().cpu().numpy()
        om.kv(1)[:, :, :n0] = vv.float().cpu().numpy()
    f0 = (torch.randn((n0, td["d_model"]), generator=torch.Generator(device="cpu").manual_seed(77)) * 0.05).float()
    g.set_context(cfg["prompt"], kv_prefilled=True)
    g.peek("feat")[:n0] = f0.cuda()
    tree = Tree(**W.draft_tree("wide"))
    ls = TreeLockStep(g, ot, od, cfg["prompt"], tree, cfg["beta"], TOL, kv_prefilled=True, temp=temp, seed=cfg["seed"], feat_prefill=f0.numpy())
    for k in (0, 1, 0):
        ls.round(k)
    assert ls.stats["max_dp"] <= TOL and ls.stats["max_dq"] <= TOL and ls.stats["max_df"] <= TOL and ls.stats["ties"] <= 1, ls.stats
    g.close()
