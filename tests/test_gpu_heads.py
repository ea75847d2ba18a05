"""GPU parity of drafter heads on the target's hidden states: the head's rows start from W_fc . [embedding ; feature of
the previous position], its own estimate feeds its next step, and the target's pass leaves the true features of the
committed rows in a table - all in lock-step with the oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import paper_2604_05417_amd as M
import workloads as W
from lockstep import LockStep

pytestmark = pytest.mark.gpu


def build_heads(cfg, T, eps, mixed=False, gamma=None):
    """K = 3 drafters: heads over target layer 0 with feature weights eps * k; `mixed` keeps drafter 1 an ordinary drafter
    with a cache of its own, so that head and non-head arms alternate in one context."""
    td, tw = cfg["target"]
    gamma = gamma or cfg["gamma"]
    drafters, heads, od = [], {}, []
    tw_np = W.to_numpy(tw)
    cache = {id(t): a for t, a in zip(tw, tw_np) if t is not None}
    for k in range(3):
        if mixed and k == 1:
            dd, dw = cfg["drafters"][1]
            fc = None
        else:
            dd, dw, fc = W.feature_head_drafter(td, tw, 0, eps * (k + 1), 300 + k)
            heads[k] = fc
        drafters.append((dd, dw))
        arrs = [None if t is None else cache.get(id(t)) for t in dw]
        arrs = [a if (a is not None or t is None) else W.to_numpy([t])[0] for a, t in zip(arrs, dw)]
        od.append(oracle.Model(dd, arrs, cfg["max_ctx"], fc=None if fc is None else W.to_numpy([fc])[0]))
    g = M.MetaSD((td, tw), drafters, gamma_max=gamma, max_ctx=cfg["max_ctx"], temperature=T, seed=cfg["seed"],
                 ucb_beta=cfg["beta"], heads=heads)
    return g, oracle.Model(td, tw_np, cfg["max_ctx"]), od


@pytest.mark.parametrize("T", [0.0, 1.0])
@pytest.mark.parametrize("mixed", [False, True])
def test_config1_drafter_heads(T, mixed):
    """Tiny fp32 configuration, 64 new tokens: logits of head and target, the feature table after every round, the
    decisions and the bookkeeping (a head keeps nothing it computed from estimated features); greedy: the target's own
    greedy continuation."""
    cfg = W.config1()
    g, ot, od = build_heads(cfg, T, 0.03, mixed)
    g.set_context(cfg["prompt"])
    ls = LockStep(g, ot, od, cfg["prompt"], cfg["gamma"], T, cfg["seed"], cfg["beta"], logit_tol=1e-4)
    B = len(cfg["prompt"]) + cfg["n_new"]
    order = [0, 1, 2, 2, 1, 0, 0, 2, 1, 1]
    while ls.l < B:
        ls.round(order[ls.t % len(order)])
    st = ls.stats
    assert st["mismatch_own"] == 0 and st["ties_own"] + st["ties_shared"] <= 1, st
    assert st["max_dp"] <= 1e-4 and st["max_dq"] <= 1e-4 and st["max_df"] <= 1e-4
    if T == 0.0:
        ref = oracle.ar_decode(oracle.Model(cfg["target"][0], W.to_numpy(cfg["target"][1]), cfg["max_ctx"]),
                               cfg["prompt"], cfg["n_new"], T=0.0)
        assert np.array_equal(ls.hist[len(cfg["prompt"]): B], ref)
    g.close()


def test_head_with_zero_feature_weight_is_the_early_exit_drafter():
    """W_fc = [I | 0]: the head's logits are those of the target's first layer under the target's norm and LM head."""
    cfg = W.config1()
    g, ot, od = build_heads(cfg, 0.0, 0.0)
    g.set_context(cfg["prompt"])
    dd, dw, _ = W.feature_head_drafter(cfg["target"][0], cfg["target"][1], 0, 0.0, 300)
    plain = oracle.Model(dd, W.to_numpy(dw), cfg["max_ctx"])
    g.draft(0, cfg["gamma"])
    Qg = g.peek("Q")[:1].cpu().numpy()
    assert np.abs(Qg[0] - plain.forward(cfg["prompt"], 0, "last")).max() <= 1e-4
    g.close()


def test_head_validation():
    cfg = W.config1()
    td, tw = cfg["target"]
    dd, dw, fc = W.feature_head_drafter(td, tw, 0, 0.01, 1)
    g = M.MetaSD((td, tw), [(dd, dw)], gamma_max=4, max_ctx=cfg["max_ctx"], temperature=0.0, seed=1)
    t = fc.cuda()
    with pytest.raises(M.MetaSDError) as e:                # the context was not created to keep features
        M.binding._check(g.L.metasd_set_drafter_head(g._h, 0, t.data_ptr()), g._h)
    assert e.value.code == -1
    g.close()
    g = M.MetaSD((td, tw), [(dd, dw)], gamma_max=4, max_ctx=cfg["max_ctx"], temperature=0.0, seed=1, heads={0: fc})
    for bad in (lambda: g.L.metasd_set_drafter_head(g._h, 1, t.data_ptr()), lambda: g.L.metasd_set_drafter_head(g._h, 0, None)):
        with pytest.raises(M.MetaSDError):
            M.binding._check(bad(), g._h)
    g.close()


@pytest.mark.parametrize("T", [0.0, 1.0])
def test_small_bf16_drafter_heads(T):
    """bf16 weights, MFMA path (pre-tiled W_fc with K = 2 d, ragged shapes): logits within the bf16 tolerance of the
    oracle run on the same bf16-rounded weights; heads and an ordinary drafter alternate."""
    cfg = W.config4(n_layers=2, ctx=45, n_new=64, K=2, d_model=256, n_heads=4, d_ffn=736, vocab=1040, dd_model=128,
                    dn_heads=2, dd_ffn=160)
    cfg["max_ctx"] = 45 + 80
    g, ot, od = build_heads(cfg, T, 0.02, mixed=True)
    g.set_context(cfg["prompt"])
    ls = LockStep(g, ot, od, cfg["prompt"], cfg["gamma"], T, cfg["seed"], cfg["beta"], logit_tol=3e-2, feat_tol=3e-2)
    order = [0, 1, 2, 2, 0]
    for _ in range(10):
        ls.round(order[ls.t % len(order)])
    assert ls.stats["max_dp"] <= 3e-2 and ls.stats["max_dq"] <= 3e-2 and ls.stats["ties_shared"] <= 1, ls.stats
    g.close()


def test_config4_7b_shape_drafter_heads_full_size():
    """7B-shape target at full size (32 layers, d 4096, FFN 11008, vocab 32000, KV context 2048) with K = 3 one-layer
    heads (W_fc [4096, 8192]) on its hidden states, T = 1: a synthetic prefix (K/V of target and heads, features) on both
    sides, then four rounds - every head once and a return to the first, which then re-reads the rows committed since
    with the target's features; logits of every row and the feature rows the target's passes add are compared."""
    cfg = W.config4(device="cuda", K=1)
    td, tw = cfg["target"]
    n0 = len(cfg["prompt"]) - 1
    drafters, heads, od = [], {}, []
    tw_np = W.to_numpy(tw)
    cache = {id(t): a for t, a in zip(tw, tw_np)}
    for k in range(3):
        dd, dw, fc = W.feature_head_drafter(td, tw, k, 0.01 * (k + 1), 300 + k)
        drafters.append((dd, dw))
        heads[k] = fc
        od.append(oracle.Model(dd, [cache[id(t)] for t in dw], cfg["max_ctx"], fc=W.to_numpy([fc])[0]))
    ot = oracle.Model(td, tw_np, cfg["max_ctx"])
    g = M.MetaSD((td, tw), drafters, gamma_max=cfg["gamma"], max_ctx=cfg["max_ctx"], temperature=1.0, seed=cfg["seed"],
                 ucb_beta=cfg["beta"], heads=heads)
    for i, (desc, kv_gpu, om) in enumerate([(td, g.kv_target, ot)] + [(dd, g.kv_drafters[k], od[k]) for k, (dd, _) in enumerate(drafters)]):
        kk, vv = W.kv_fill(desc, n0, cfg["kv_seed"] + i, device="cuda")
        kv_gpu[:, 0, :, :n0] = kk
        kv_gpu[:, 1, :, :n0] = vv
        om.kv(0)[:, :, :n0] = kk.float().cpu().numpy()
        om.kv(1)[:, :, :n0] = vv.float().cpu().numpy()
    gen = torch.Generator(device="cpu").manual_seed(77)
    f0 = (torch.randn((n0, td["d_model"]), generator=gen) * 0.05).float()
    g.set_context(cfg["prompt"], kv_prefilled=True)
    g.peek("feat")[:n0] = f0.cuda()
    ls = LockStep(g, ot, od, cfg["prompt"], cfg["gamma"], 1.0, cfg["seed"], cfg["beta"], logit_tol=3e-2, kv_prefilled=True,
                  feat_tol=3e-2, feat_prefill=f0.numpy())
    for k in (0, 1, 2, 0):
        ls.round(k)
    st = ls.stats
    assert st["max_dp"] <= 3e-2 and st["max_dq"] <= 3e-2 and st["ties_shared"] <= 1, st
    g.close()


@pytest.mark.parametrize("T", [0.0, 1.0])
def test_head_catch_up_over_a_long_backlog(T):
    """A head that sat out many rounds re-reads a backlog longer than one 16-row block (the feature rows of every block come
    from the table the target's passes filled meanwhile), and a head chosen many times in a row re-reads the rows of its
    own previous round every time; fp32, lock-step."""
    cfg = W.config1()
    cfg["max_ctx"] = 16 + 120
    g, ot, od = build_heads(cfg, T, 0.03, mixed=True)
    g.set_context(cfg["prompt"])
    ls = LockStep(g, ot, od, cfg["prompt"], cfg["gamma"], T, cfg["seed"], cfg["beta"], logit_tol=1e-4)
    order = [1] * 9 + [0] + [2] * 6 + [0, 0, 0, 2]
    backlog = []
    for k in order:
        if k != 1:
            backlog.append(ls.l - ls.c[k])
        ls.round(k)
    st = ls.stats
    assert max(backlog) > 16, backlog
    assert st["mismatch_own"] == 0 and st["ties_own"] + st["ties_shared"] <= 1, st
    assert st["max_dp"] <= 1e-4 and st["max_dq"] <= 1e-4 and st["max_df"] <= 1e-4
    g.close()
