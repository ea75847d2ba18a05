"""The oracle's MetaSD loop (Alg. 1 / Alg. 2 around Alg. 3 rounds) on the tiny configuration."""
import numpy as np
import torch
import pytest

import oracle
import workloads as W


@pytest.fixture(scope="module")
def c1():
    cfg = W.config1()
    td, tw = cfg["target"]
    cfg["tw_np"] = W.to_numpy(tw)
    cfg["dw_np"] = [W.to_numpy(dw) for _, dw in cfg["drafters"]]
    return cfg


def models(cfg):
    td, _ = cfg["target"]
    T = oracle.Model(td, cfg["tw_np"], cfg["max_ctx"])
    D = [oracle.Model(dd, w, cfg["max_ctx"]) for (dd, _), w in zip(cfg["drafters"], cfg["dw_np"])]
    return T, D


def test_greedy_sd_equals_target_only_greedy(c1):
    """Speculative decoding is lossless (Sec. 2.1, Alg. 3): with T = 0 every drafter, also a
    badly aligned one, must reproduce plain greedy decoding of the target token for token."""
    T, _ = models(c1)
    ref = oracle.ar_decode(T, c1["prompt"], c1["n_new"], T=0.0)
    accs = []
    for pol in (None, 0, 1, 2):
        T, D = models(c1)
        out = oracle.generate(T, D, c1["prompt"], c1["n_new"], c1["gamma"], 0.0, c1["seed"], c1["beta"],
                              policy=None if pol is None else (lambda t, a=pol: a))
        assert np.array_equal(out["tokens"], ref), pol
        # accounting: B = tau + sum N_acc (proof of the stopping-time lemma), before truncation
        tau = len(out["rounds"])
        assert out["total_len"] - len(c1["prompt"]) == tau + sum(r["n_acc"] for r in out["rounds"])
        assert out["t"] == tau and out["n"].sum() == tau
        accs.append(np.mean([r["n_acc"] for r in out["rounds"]]))
    # drafter 0 is the exact early exit; drafter 2 carries the largest head noise
    assert accs[1] >= accs[3]


def test_initial_sweep_visits_arms_in_order(c1):
    T, D = models(c1)
    out = oracle.generate(T, D, c1["prompt"], 24, c1["gamma"], 1.0, c1["seed"], c1["beta"])
    assert [r["k"] for r in out["rounds"][:3]] == [0, 1, 2]
    assert all(np.isnan(r["scores"]).all() for r in out["rounds"][:3])
    assert all(0 <= r["reward"] <= 1 for r in out["rounds"])
    assert len(out["tokens"]) == 24 and out["tokens"].min() >= 0 and out["tokens"].max() < 512


def test_sampling_run_is_reproducible_and_seed_dependent(c1):
    outs = []
    for seed in (1, 1, 2):
        T, D = models(c1)
        outs.append(oracle.generate(T, D, c1["prompt"], 32, c1["gamma"], 1.0, seed, c1["beta"], reward="BD")["tokens"])
    assert np.array_equal(outs[0], outs[1]) and not np.array_equal(outs[0], outs[2])


def test_drafter_catch_up_after_switch(c1):
    """A drafter that sat out several rounds first consumes the tokens it missed: its logits for
    the next position equal those of a fresh copy fed the whole committed sequence."""
    T, D = models(c1)
    out = oracle.generate(T, D, c1["prompt"], 20, c1["gamma"], 0.0, c1["seed"], c1["beta"],
                          policy=lambda t: 0 if t < 4 else 1, keep_logits=True)
    st = out["state"]
    r = next(r for r in out["rounds"] if r["k"] == 1)
    fresh = oracle.Model(c1["drafters"][1][0], c1["dw_np"][1], c1["max_ctx"])
    want = fresh.forward(st.hist[: r["l_before"]], 0, "last")
    assert np.abs(want - r["Q"][0]).max() < 1e-5


def shared_models(cfg):
    """Target and early-exit drafters that keep no cache of their own (they read and write the target's)."""
    td, _ = cfg["target"]
    T = oracle.Model(td, cfg["tw_np"], cfg["max_ctx"])
    D = [oracle.Model(dd, w, cfg["max_ctx"], share_kv_with=T) for (dd, _), w in zip(cfg["drafters"], cfg["dw_np"])]
    return T, D


@pytest.mark.parametrize("T", [0.0, 1.0])
def test_shared_cache_drafters_equal_own_cache_drafters(c1, T):
    """An early-exit drafter runs the target's first layers, so the K/V it needs at committed positions are the
    numbers the target's cache already holds (same weights, same inputs, and the oracle's arithmetic does not
    depend on how rows are grouped into blocks).  Reading them there instead of recomputing them when the drafter
    is switched in must therefore change nothing: the same drafter logits bit for bit, the same tokens, the same
    arms - over a whole generation in which the bandit switches drafters."""
    Ta, Da = models(c1)
    a = oracle.generate(Ta, Da, c1["prompt"], c1["n_new"], c1["gamma"], T, c1["seed"], c1["beta"], keep_logits=True)
    Tb, Db = shared_models(c1)
    b = oracle.generate(Tb, Db, c1["prompt"], c1["n_new"], c1["gamma"], T, c1["seed"], c1["beta"], keep_logits=True)
    assert np.array_equal(a["tokens"], b["tokens"])
    assert [r["k"] for r in a["rounds"]] == [r["k"] for r in b["rounds"]]
    assert len({r["k"] for r in a["rounds"]}) == 3                       # every drafter was switched in at least once
    for ra, rb in zip(a["rounds"], b["rounds"]):
        assert np.abs(ra["Q"] - rb["Q"]).max() <= 1e-5 and np.abs(ra["P"] - rb["P"]).max() <= 1e-5
        assert np.array_equal(ra["Q"], rb["Q"]) and np.array_equal(ra["P"], rb["P"])
        assert np.array_equal(ra["d"], rb["d"]) and ra["n_acc"] == rb["n_acc"] and ra["token"] == rb["token"]
    # and a drafter whose layers are NOT the owner's first layers cannot be created on its cache
    td = dict(c1["target"][0])
    td["n_layers"] = 3
    with pytest.raises(MemoryError):
        oracle.Model(td, c1["tw_np"][:1] + c1["tw_np"][1:10] * 3 + c1["tw_np"][-2:], c1["max_ctx"], share_kv_with=Tb)


def test_shared_cache_greedy_is_lossless(c1):
    """Losslessness (paragraph after Alg. 3) holds for the shared-cache strategy as well: greedy speculative decoding
    with drafters that read the target's cache reproduces target-only greedy decoding token for token."""
    T0, _ = models(c1)
    ref = oracle.ar_decode(T0, c1["prompt"], c1["n_new"], T=0.0)
    for arm in (0, 2):
        T, D = shared_models(c1)
        out = oracle.generate(T, D, c1["prompt"], c1["n_new"], c1["gamma"], 0.0, c1["seed"], c1["beta"], policy=lambda t, a=arm: a)
        assert np.array_equal(out["tokens"], ref)


# ---------------------------------------------------------------- streaming drafter caches (sinks + window)

def _stream_models(cfg, stream, share=False):
    T = oracle.Model(cfg["target"][0], W.to_numpy(cfg["target"][1]), cfg["max_ctx"])
    D = [oracle.Model(dd, W.to_numpy(dw), cfg["max_ctx"], stream=stream) for dd, dw in cfg["drafters"]]
    return T, D


def test_streaming_cache_with_a_window_as_long_as_the_text_is_the_plain_cache():
    """Sinks + window covering everything: the mask is the causal mask and nothing is skipped, so the rounds are those of
    drafters with full caches, logit for logit."""
    cfg = W.config1()
    T, D = _stream_models(cfg, None)
    a = oracle.generate(T, D, cfg["prompt"], 40, cfg["gamma"], 1.0, cfg["seed"], cfg["beta"], keep_logits=True)
    T, D = _stream_models(cfg, (3, cfg["max_ctx"]))
    b = oracle.generate(T, D, cfg["prompt"], 40, cfg["gamma"], 1.0, cfg["seed"], cfg["beta"], keep_logits=True)
    assert np.array_equal(a["tokens"], b["tokens"])
    for ra, rb in zip(a["rounds"], b["rounds"]):
        assert np.array_equal(ra["Q"], rb["Q"]) and np.array_equal(ra["P"], rb["P"])


def test_streaming_row_sees_sinks_and_window_only():
    """The logits of a streaming drafter at position p are those of a fresh model that was fed only the sink tokens and
    the window's tokens, each at its original position (compact cache slots, same rotations) - attention over the visible
    set, computed the other way round."""
    from oracle.loop import stream_catch_up
    cfg = W.config1()
    dd, dw = cfg["drafters"][1]
    S, Wn = 2, 5
    rng = np.random.default_rng(4)
    toks = rng.integers(0, 512, 40).astype(np.int32)
    A = oracle.Model(dd, W.to_numpy(dw), cfg["max_ctx"], stream=(S, Wn))
    for l in (1, 2, 4, 9, 23, 40):                       # shorter than the sinks, inside the window, far beyond it
        A2 = oracle.Model(dd, W.to_numpy(dw), cfg["max_ctx"], stream=(S, Wn))
        q, a = stream_catch_up(A2, toks, 0, l, 0)
        vis = sorted(set(range(min(S, l))) | set(range(max(0, l - Wn), l)))
        assert a == (max(min(S, l), l - Wn) if l - Wn > min(S, l) else 0)
        B = oracle.Model(dd, W.to_numpy(dw), cfg["max_ctx"])
        allow = np.zeros((len(vis), B.max_ctx), np.uint8)
        for r, p in enumerate(vis):
            lo = max(a, p - Wn + 1) if p >= S else 0
            for r2, p2 in enumerate(vis[: r + 1]):
                if p2 < S or p2 >= lo:
                    allow[r, r2] = 1
        ref = B.forward_rows(toks[vis], np.arange(len(vis)), vis, allow)[-1]
        assert np.array_equal(q, ref), l
    del A


@pytest.mark.parametrize("stream", [(2, 6), (0, 3), (4, 12)])
def test_streaming_caches_keep_greedy_decoding_lossless(stream):
    """Whatever the drafters' cache strategy, greedy MetaSD emits the target's own greedy continuation; arms forced so that
    every drafter sits out longer than its window and comes back (the skipped backlog must never be attended to)."""
    cfg = W.config1()
    T, D = _stream_models(cfg, stream)
    order = [0, 0, 1, 1, 1, 1, 2, 2, 2, 2, 0, 1, 2, 0, 0, 0, 1]
    out = oracle.generate(T, D, cfg["prompt"], cfg["n_new"], cfg["gamma"], 0.0, cfg["seed"], cfg["beta"], policy=lambda r: order[r % len(order)])
    ref = oracle.ar_decode(oracle.Model(cfg["target"][0], W.to_numpy(cfg["target"][1]), cfg["max_ctx"]), cfg["prompt"], cfg["n_new"], T=0.0)
    assert np.array_equal(out["tokens"], ref)
    st = out["state"]
    assert st.a is not None and max(st.a) > 0                # some backlog was skipped


# ---------------------------------------------------------------- drafter heads on the target's hidden states

def _head_models(cfg, eps, layer=0):
    T = oracle.Model(cfg["target"][0], W.to_numpy(cfg["target"][1]), cfg["max_ctx"])
    D = []
    for k in range(3):
        dd, dw, fc = W.feature_head_drafter(cfg["target"][0], cfg["target"][1], layer, eps * k if eps else 0.0, 300 + k)
        D.append(oracle.Model(dd, W.to_numpy(dw), cfg["max_ctx"], fc=W.to_numpy([fc])[0]))
    return T, D


def test_feature_is_the_residual_stream_before_the_final_norm():
    """logits = LM head . RMSNorm(feature) . gain, recomputed here with numpy from the returned features."""
    cfg = W.config1()
    td, tw = cfg["target"]
    T = oracle.Model(td, W.to_numpy(tw), cfg["max_ctx"])
    P, H = T.forward_hidden(cfg["prompt"][:9], 0, "all")
    g = tw[-2].double().numpy()
    head = tw[-1].double().numpy()
    x = H.astype(np.float64)
    x = x / np.sqrt((x * x).mean(axis=1, keepdims=True) + td["rms_eps"]) * g
    assert np.abs(x.astype(np.float32).astype(np.float64) @ head.T - P).max() < 2e-5
    assert np.array_equal(T.forward(cfg["prompt"][9:12], 9, "all"), T.forward_hidden(cfg["prompt"][9:12], 9, "all")[0])


def test_head_that_ignores_the_features_is_the_early_exit_drafter():
    """W_fc = [I | 0]: the head's rows start from the token embedding, so it is the target's first layer with the target's
    norm and LM head - the early-exit drafter after one layer, logit for logit, and the whole generation is the same (the
    head re-reads the committed tokens of the last round, which changes nothing when the features carry no weight)."""
    cfg = W.config1()
    td, tw = cfg["target"]
    T, D = _head_models(cfg, 0.0)
    a = oracle.generate(T, D, cfg["prompt"], 48, cfg["gamma"], 1.0, cfg["seed"], cfg["beta"], keep_logits=True)
    T2 = oracle.Model(td, W.to_numpy(tw), cfg["max_ctx"])
    D2 = []
    for k in range(3):
        dd, dw = W.early_exit_drafter(td, tw, 1, 0.0, 100 + k)
        D2.append(oracle.Model(dd, W.to_numpy(dw), cfg["max_ctx"]))
    b = oracle.generate(T2, D2, cfg["prompt"], 48, cfg["gamma"], 1.0, cfg["seed"], cfg["beta"], keep_logits=True)
    assert np.array_equal(a["tokens"], b["tokens"])
    for ra, rb in zip(a["rounds"], b["rounds"]):
        assert np.array_equal(ra["Q"], rb["Q"]) and ra["n_acc"] == rb["n_acc"]
    assert max(r["n_acc"] for r in a["rounds"]) >= 1


def test_head_that_passes_the_feature_through_gives_the_targets_logits_of_that_position():
    """W_fc = [0 | I] and a layer that adds nothing (zero output projections): the head's estimate is the feature it was
    given, so its logits at position p are the target's logits of position p - 1 - the concatenation order, the feature
    offset and the use of the target's norm and head in one check."""
    cfg = W.config1()
    td, tw = cfg["target"]
    T = oracle.Model(td, W.to_numpy(tw), cfg["max_ctx"])
    P, H = T.forward_hidden(cfg["prompt"][:10], 0, "all")
    dd, dw, _ = W.feature_head_drafter(td, tw, 0, 0.0, 1)
    dw = list(dw)
    dw[5] = torch.zeros_like(dw[5])          # wo
    dw[9] = torch.zeros_like(dw[9])          # w_down
    d = td["d_model"]
    fc = torch.cat([torch.zeros(d, d), torch.eye(d)], dim=1).contiguous()
    Hd = oracle.Model(dd, W.to_numpy(dw), cfg["max_ctx"], fc=fc.numpy())
    feats = np.zeros((10, d), np.float32)
    feats[1:] = H[:9]
    Q, est = Hd.forward_hidden(cfg["prompt"][:10], 0, "all", feats=feats)
    assert np.array_equal(est, feats)
    assert np.array_equal(Q[1:], P[:9])


@pytest.mark.parametrize("T", [0.0, 1.0])
def test_generation_with_drafter_heads(T):
    """Greedy: the target's own greedy continuation whatever the heads do; any T: the features kept along the way are the
    target's features of the committed text (a fresh pass over it gives them again), and tokens do get accepted."""
    cfg = W.config1()
    td, tw = cfg["target"]
    Tm, D = _head_models(cfg, 0.05)
    order = [0, 1, 2, 2, 1, 0, 0, 2]
    out = oracle.generate(Tm, D, cfg["prompt"], cfg["n_new"], cfg["gamma"], T, cfg["seed"], cfg["beta"], policy=lambda r: order[r % len(order)])
    st = out["state"]
    if T == 0.0:
        ref = oracle.ar_decode(oracle.Model(td, W.to_numpy(tw), cfg["max_ctx"]), cfg["prompt"], cfg["n_new"], T=0.0)
        assert np.array_equal(out["tokens"], ref)
    fresh = oracle.Model(td, W.to_numpy(tw), cfg["max_ctx"])
    _, H = fresh.forward_hidden(st.hist[: st.l - 1], 0, None)
    assert np.array_equal(st.feat[: st.l - 1], H)
    assert max(r["n_acc"] for r in out["rounds"]) >= 1
    assert all(c <= st.l - 1 for c in st.c)
