"""GPU parity of the full MetaSD loop (select -> draft -> verify -> accept -> update) against the
oracle, teacher-forced round by round (see lockstep.py), through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import paper_2604_05417_amd as M
import workloads as W
from lockstep import LockStep

pytestmark = pytest.mark.gpu


def build_pair(cfg, T, reward="BE", gamma=None, device="cuda", stream=None):
    td, tw = cfg["target"]
    gamma = gamma or cfg["gamma"]
    g = M.MetaSD((td, tw), cfg["drafters"], gamma_max=gamma, max_ctx=cfg["max_ctx"], temperature=T, seed=cfg["seed"],
                 ucb_beta=cfg["beta"], reward=reward, stream=stream)
    tw_np = W.to_numpy(tw)
    cache = {id(t): a for t, a in zip(tw, tw_np) if t is not None}
    ot = oracle.Model(td, tw_np, cfg["max_ctx"])
    od = []
    for dd, dw in cfg["drafters"]:
        arrs = [None if t is None else cache.get(id(t)) for t in dw]
        arrs = [a if (a is not None or t is None) else W.to_numpy([t])[0] for a, t in zip(arrs, dw)]
        od.append(oracle.Model(dd, arrs, cfg["max_ctx"], stream=stream))
    return g, ot, od


@pytest.mark.parametrize("T,reward", [(0.0, "BE"), (1.0, "BE"), (0.7, "BD")])
def test_config1_full_loop(T, reward):
    """Tiny fp32 configuration: 2-layer GELU target, K = 3 early-exit drafters, gamma = 4, 64 new tokens."""
    cfg = W.config1()
    g, ot, od = build_pair(cfg, T, reward)
    g.set_context(cfg["prompt"])
    ls = LockStep(g, ot, od, cfg["prompt"], cfg["gamma"], T, cfg["seed"], cfg["beta"], logit_tol=1e-4, reward=reward)
    B = len(cfg["prompt"]) + cfg["n_new"]
    while ls.l < B:
        ls.round()
    st = ls.stats
    assert st["mismatch_own"] == 0 and st["ties_own"] + st["ties_shared"] <= 1, st
    assert st["max_dp"] <= 1e-4 and st["max_dq"] <= 1e-4
    assert st["arms"][:3] == [0, 1, 2]
    if T == 0.0:
        assert st["ties_own"] == 0 and st["ties_shared"] == 0
        # lossless: the committed tokens equal plain greedy decoding of the target
        ref = oracle.ar_decode(oracle.Model(cfg["target"][0], W.to_numpy(cfg["target"][1]), cfg["max_ctx"]),
                               cfg["prompt"], cfg["n_new"], T=0.0)
        assert np.array_equal(ls.hist[len(cfg["prompt"]): B], ref)
    g.close()


def test_call_order_and_limits():
    cfg = W.config1()
    g, _, _ = build_pair(cfg, 1.0)
    with pytest.raises(M.MetaSDError) as e:
        g.draft(0, 4)                                      # no context yet
    assert e.value.code == -3
    g.set_context(cfg["prompt"])
    for bad in (lambda: g.verify(4), lambda: g.accept(4)):
        with pytest.raises(M.MetaSDError) as e:
            bad()
        assert e.value.code == -3
    with pytest.raises(M.MetaSDError) as e:
        g.draft(3, 4)                                      # K = 3
    assert e.value.code == -1
    with pytest.raises(M.MetaSDError) as e:
        g.draft(0, 5)                                      # gamma_max = 4
    assert e.value.code == -1
    g.draft(1, 2)
    with pytest.raises(M.MetaSDError):
        g.verify(3)                                        # gamma differs from the draft
    g.verify(2)
    n, tok, mask, bd = g.accept(2)
    assert 0 <= n <= 2 and 0 <= tok < 512 and 0.0 <= bd <= 1.0
    with pytest.raises(M.MetaSDError) as e:
        g.set_context(np.zeros(cfg["max_ctx"], np.int32))  # no room for a round
    assert e.value.code == -2
    with pytest.raises(M.MetaSDError):
        g.set_context(np.array([1, 2, 600], np.int32))     # token outside the vocabulary
    g.set_context(cfg["prompt"][:1])                       # a one-token prompt needs no prefill
    g.round(4)
    g.close()


def test_runs_out_of_context_cleanly():
    cfg = W.config1()
    cfg["max_ctx"] = 16 + 12
    g, _, _ = build_pair(cfg, 0.0)
    g.set_context(cfg["prompt"])
    with pytest.raises(M.MetaSDError) as e:
        for _ in range(20):
            g.round(4)
    assert e.value.code == -2
    g.close()


@pytest.mark.parametrize("T", [0.0, 1.0])
def test_smallest_sizes_one_drafter_one_draft_one_prompt_token(T):
    """The degenerate ends of the ranges: K = 1 (Alg. 2's index then only ever has one arm; its bonus term is finite
    from the first decision on), gamma = 1 (a two-row verification block), a one-token prompt (nothing to prefill);
    20 rounds in lock-step with the oracle."""
    cfg = W.config1()
    cfg["drafters"] = cfg["drafters"][:1]
    cfg["prompt"] = cfg["prompt"][:1]
    g, ot, od = build_pair(cfg, T, gamma=1)
    g.set_context(cfg["prompt"])
    ls = LockStep(g, ot, od, cfg["prompt"], 1, T, cfg["seed"], cfg["beta"], logit_tol=1e-4)
    for _ in range(20):
        ls.round()
    st = ls.stats
    assert st["mismatch_own"] == 0 and st["ties_own"] + st["ties_shared"] <= 1 and st["max_dp"] <= 1e-4 and st["max_dq"] <= 1e-4, st
    assert set(st["arms"]) == {0}
    g.close()


@pytest.mark.parametrize("T", [0.0, 1.0])
@pytest.mark.parametrize("stream", [(2, 6), (0, 3)])
def test_config1_streaming_drafter_caches(T, stream):
    """The tiny fp32 loop with streaming drafter caches (the plain attention kernel with the sink + window mask): 64 new
    tokens in lock-step, arms forced so that drafters sit out longer than their window; greedy: the target's own greedy
    continuation."""
    cfg = W.config1()
    g, ot, od = build_pair(cfg, T, stream=stream)
    g.set_context(cfg["prompt"])
    ls = LockStep(g, ot, od, cfg["prompt"], cfg["gamma"], T, cfg["seed"], cfg["beta"], logit_tol=1e-4)
    B = len(cfg["prompt"]) + cfg["n_new"]
    order = [0, 0, 1, 1, 1, 1, 2, 2, 2, 2, 0, 1, 2, 0, 0, 0, 1]
    while ls.l < B:
        ls.round(order[ls.t % len(order)])
    st = ls.stats
    assert st["mismatch_own"] == 0 and st["ties_own"] + st["ties_shared"] <= 1, st
    assert st["max_dp"] <= 1e-4 and st["max_dq"] <= 1e-4 and max(ls.a) > 0
    if T == 0.0:
        ref = oracle.ar_decode(oracle.Model(cfg["target"][0], W.to_numpy(cfg["target"][1]), cfg["max_ctx"]),
                               cfg["prompt"], cfg["n_new"], T=0.0)
        assert np.array_equal(ls.hist[len(cfg["prompt"]): B], ref)
    g.close()
